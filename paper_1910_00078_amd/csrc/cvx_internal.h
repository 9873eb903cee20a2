// Internal declarations shared by the host dispatch code and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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
    KID_COUNT
};

struct KernelChoice {
    KernelId id;
    const char* name;        // static string
};

KernelChoice select_kernel(const ConvArgs& a, int policy);

hipError_t launch_direct(const ConvArgs& a, hipStream_t s);
bool igemm_supported(const ConvArgs& a, const char** variant_name);
hipError_t launch_igemm(const ConvArgs& a, hipStream_t s);
bool stem_supported(const ConvArgs& a, const char** variant_name);
hipError_t launch_stem(const ConvArgs& a, hipStream_t s);
bool pointwise_supported(const ConvArgs& a, const char** variant_name);
hipError_t launch_pointwise(const ConvArgs& a, hipStream_t s);

hipError_t launch_bias_add(void* y, const void* bias, int dtype, int bias_f32, int N, int K, int HW, hipStream_t s);
hipError_t launch_activation(void* y, int dtype, int act, float alpha, long long count, hipStream_t s);

}  // namespace cvx
