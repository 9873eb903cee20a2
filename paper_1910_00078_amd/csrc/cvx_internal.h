// Internal declarations shared by the host dispatch code and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace cvx {

enum : int { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2 };
enum : int { ACT_IDENTITY = 0, ACT_RELU = 1, ACT_LEAKY_RELU = 2, ACT_TANH = 3, ACT_LOGISTIC = 4 };

// Everything a kernel needs to know about one forward convolution.  Plain data, passed by value.
struct ConvArgs {
    const void* x;
    const void* w;
    const void* bias;        // nullable
    void* y;
    const float* bn_scale;   // nullable: all four set or none
    const float* bn_shift;
    const float* bn_mean;
    const float* bn_var;
    float bn_eps;
    float alpha;
    int dtype;               // DT_* of x, w, y
    int bias_f32;            // 1: bias is fp32, 0: bias has the data dtype
    int act;
    int N, C, H, W, K, R, S, Ho, Wo;
    int pad_h, pad_w, stride_h, stride_w, dil_h, dil_w, groups;
};

// Which kernel family serves a problem.
enum KernelId : int {
    KID_DIRECT = 0,          // one thread per output, any parameters
    KID_IGEMM,               // MFMA implicit GEMM, 16-bit types
    KID_STEM,                // low-channel strided direct-MFMA kernel
    KID_POINTWISE,           // persistent streaming kernel for 1x1 filters
    KID_TILED_F32,           // LDS-tiled fp32 kernel on the fp32 matrix instruction
    KID_COUNT
};

// What a kernel choice may depend on besides the problem itself.  Nothing here is a data pointer: a
// plan made once serves every later call with the same problem and environment.
struct PlanEnv {
    int cus;                  // compute units of the device
    int policy;               // 0: automatic choice, 1: generic direct kernel only
    bool aligned16;           // x, w and y are all 16-byte aligned
    const char* pin;          // developer pin "<variant>[,<NB>,<TH>]", or nullptr
};

// The host's decision for one problem: kernel, geometry and launch shape.
struct LaunchPlan {
    KernelId id;
    const char* name;         // static string
    int variant;              // index into the family's variant table
    unsigned grid_x, grid_y, block;
    int lds;                  // dynamic LDS bytes
    alignas(8) unsigned char geom[288];   // the family's geometry struct (a kernel argument)
};

// Each family: plan() returns false if it does not serve the problem; launch() enqueues what plan() decided.
bool igemm_plan(const ConvArgs& a, const PlanEnv& env, LaunchPlan* out);
hipError_t igemm_launch(const ConvArgs& a, const LaunchPlan& p, hipStream_t s);
bool stem_plan(const ConvArgs& a, const PlanEnv& env, LaunchPlan* out);
hipError_t stem_launch(const ConvArgs& a, const LaunchPlan& p, hipStream_t s);
bool pointwise_plan(const ConvArgs& a, const PlanEnv& env, LaunchPlan* out);
hipError_t pointwise_launch(const ConvArgs& a, const LaunchPlan& p, hipStream_t s);
bool tiled_f32_plan(const ConvArgs& a, const PlanEnv& env, LaunchPlan* out);
hipError_t tiled_f32_launch(const ConvArgs& a, const LaunchPlan& p, hipStream_t s);
bool direct_plan(const ConvArgs& a, const PlanEnv& env, LaunchPlan* out);
hipError_t direct_launch(const ConvArgs& a, const LaunchPlan& p, hipStream_t s);

// Raises the dynamic-LDS limit of every kernel of a family (once per process; not a stream operation).
hipError_t igemm_prepare();
hipError_t stem_prepare();
hipError_t pointwise_prepare();
hipError_t tiled_f32_prepare();

// The problem -> kernel choice (the job the paper gives its solvers, Sec. III-A).  False only if a
// developer pin names a kernel that cannot run the problem.
bool make_plan(const ConvArgs& a, const PlanEnv& env, LaunchPlan* out);
hipError_t launch_plan(const ConvArgs& a, const LaunchPlan& p, hipStream_t s);

hipError_t launch_bias_add(void* y, const void* bias, int dtype, int bias_f32, int N, int K, int HW, hipStream_t s);
hipError_t launch_activation(void* y, int dtype, int act, float alpha, long long count, hipStream_t s);

}  // namespace cvx
