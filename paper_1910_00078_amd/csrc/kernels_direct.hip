// Generic direct forward convolution: one thread per output element, any filter size, padding,
// stride, dilation and group count, all three data types, fp32 accumulation, fused epilogue.
// This is the correctness net behind the specialised kernels (the "direct" family of Sec. IV-A of
// the MIOpen paper in its plainest form), plus the separate bias / activation operators that the
// unfused path of Sec. V uses.
#include "cvx_device.h"

namespace cvx {

// CS = 1: one thread per output.  CS = 8: eight neighbouring lanes share an output, each taking every
// eighth channel, and add their partial sums with three lane exchanges: small problems are a chain of
// dependent loads per thread, and this cuts the chain by eight.
template <int DT, int CS>
__global__ void __launch_bounds__(256) direct_conv_kernel(ConvArgs a)
{
    warm_kernel_arguments<sizeof(ConvArgs)>();
    const long long total = (long long)a.N * a.K * a.Ho * a.Wo;
    const int cg = a.C / a.groups;
    const int kg = a.K / a.groups;
    const bool has_bn = a.bn_scale != nullptr;
    const long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int part = (int)(tid % CS);
    for (long long o = tid / CS; o < total; o += (long long)gridDim.x * blockDim.x / CS) {
        const int q = (int)(o % a.Wo);
        long long t = o / a.Wo;
        const int p = (int)(t % a.Ho);
        t /= a.Ho;
        const int k = (int)(t % a.K);
        const int n = (int)(t / a.K);
        const int c0 = (k / kg) * cg;
        const int h0 = p * a.stride_h - a.pad_h;
        const int w0 = q * a.stride_w - a.pad_w;
        float acc = 0.0f;
        for (int c = part; c < cg; c += CS) {
            const size_t xbase = ((size_t)n * a.C + (c0 + c)) * a.H * a.W;
            const size_t wbase = ((size_t)k * cg + c) * a.R * a.S;
            for (int r = 0; r < a.R; ++r) {
                const int h = h0 + r * a.dil_h;
                if (h < 0 || h >= a.H) continue;
                for (int s = 0; s < a.S; ++s) {
                    const int wv = w0 + s * a.dil_w;
                    if (wv < 0 || wv >= a.W) continue;
                    acc = fmaf(Elem<DT>::load(a.x, xbase + (size_t)h * a.W + wv),
                               Elem<DT>::load(a.w, wbase + (size_t)r * a.S + s), acc);
                }
            }
        }
        if constexpr (CS > 1) {
            // the CS lanes of an output are neighbours in one wave and reach this point together
#pragma unroll
            for (int d = 1; d < CS; d <<= 1) acc += __shfl_xor(acc, d);
            if (part != 0) continue;
        }
        const ChannelAffine ca = channel_affine<DT>(a, k);
        Elem<DT>::store(a.y, (size_t)o, finish(acc, ca, has_bn, a.act, a.alpha));
    }
}

bool direct_plan(const ConvArgs& a, const PlanEnv&, LaunchPlan* out)
{
    const long long total = (long long)a.N * a.K * a.Ho * a.Wo;
    const bool split = total <= 32768 && a.C / a.groups >= 8;      // latency-bound sizes
    long long blocks = (total * (split ? 8 : 1) + 255) / 256;
    if (blocks > (1 << 20)) blocks = 1 << 20;           // grid-stride loop covers the rest
    out->id = KID_DIRECT;
    out->name = a.dtype == DT_F32 ? "direct_f32" : a.dtype == DT_F16 ? "direct_f16" : "direct_bf16";
    out->variant = split ? 8 : 1;
    out->grid_x = (unsigned)blocks;
    out->grid_y = 1;
    out->block = 256;
    out->lds = 0;
    return true;
}

hipError_t direct_launch(const ConvArgs& a, const LaunchPlan& p, hipStream_t s)
{
    const dim3 grid(p.grid_x), block(p.block);
    const bool split = p.variant == 8;
#define CVX_LAUNCH_DIRECT(DT)                                                                   \
    do {                                                                                        \
        if (split) hipLaunchKernelGGL((direct_conv_kernel<DT, 8>), grid, block, 0, s, a);       \
        else hipLaunchKernelGGL((direct_conv_kernel<DT, 1>), grid, block, 0, s, a);             \
    } while (0)
    switch (a.dtype) {
    case DT_F32:  CVX_LAUNCH_DIRECT(DT_F32); break;
    case DT_F16:  CVX_LAUNCH_DIRECT(DT_F16); break;
    case DT_BF16: CVX_LAUNCH_DIRECT(DT_BF16); break;
    default: return hipErrorInvalidValue;
    }
#undef CVX_LAUNCH_DIRECT
    return hipGetLastError();
}

// ---- unfused element-wise operators --------------------------------------------------------------
// Each thread handles 16 bytes (8 fp16/bf16 or 4 fp32 elements) per step when y is 16-byte aligned
// (`vec` = elements per vector, else 1); the bias kernel also needs HW to be a multiple of the
// vector so that a vector never straddles two channels.  Elements past the last whole vector are
// done one by one by the first threads.
typedef uint32_t ew_u32x4 __attribute__((ext_vector_type(4)));

template <int DT, typename F>
__device__ __forceinline__ void ew_apply_vector(void* y, long long v, F&& f)
{
    ew_u32x4 q = ((const ew_u32x4*)y)[v];
    if constexpr (DT == DT_F32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) q[e] = __float_as_uint(f(__uint_as_float(q[e])));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float lo = f(bits16_to_f32<DT>((uint16_t)(q[e] & 0xffffu)));
            const float hi = f(bits16_to_f32<DT>((uint16_t)(q[e] >> 16)));
            q[e] = (uint32_t)f32_to_bits16<DT>(lo) | ((uint32_t)f32_to_bits16<DT>(hi) << 16);
        }
    }
    ((ew_u32x4*)y)[v] = q;
}

template <int DT>
__global__ void __launch_bounds__(256) bias_add_kernel(void* y, const void* bias, int bias_f32,
                                                        int K, int HW, long long total, int vec)
{
    const long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x, nthreads = (long long)gridDim.x * blockDim.x;
    const long long nvec = vec > 1 ? total / vec : 0;
    for (long long v = tid; v < nvec; v += nthreads) {
        const int k = (int)(((v * vec) / HW) % K);
        const float b = bias_f32 ? ((const float*)bias)[k] : Elem<DT>::load(bias, k);
        ew_apply_vector<DT>(y, v, [b](float t) { return t + b; });
    }
    for (long long i = nvec * vec + tid; i < total; i += nthreads) {
        const int k = (int)((i / HW) % K);
        const float b = bias_f32 ? ((const float*)bias)[k] : Elem<DT>::load(bias, k);
        Elem<DT>::store(y, (size_t)i, Elem<DT>::load(y, (size_t)i) + b);
    }
}

template <int DT>
__global__ void __launch_bounds__(256) activation_kernel(void* y, int act, float alpha, long long total, int vec)
{
    const long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x, nthreads = (long long)gridDim.x * blockDim.x;
    const long long nvec = vec > 1 ? total / vec : 0;
    if (act == ACT_RELU) {
        for (long long v = tid; v < nvec; v += nthreads) ew_apply_vector<DT>(y, v, [](float t) { return fmaxf(t, 0.0f); });
    } else {
        for (long long v = tid; v < nvec; v += nthreads) ew_apply_vector<DT>(y, v, [act, alpha](float t) { return activate(t, act, alpha); });
    }
    for (long long i = nvec * vec + tid; i < total; i += nthreads)
        Elem<DT>::store(y, (size_t)i, activate(Elem<DT>::load(y, (size_t)i), act, alpha));
}

static int ew_vector(const void* y, int dtype)
{
    return ((uintptr_t)y & 15) ? 1 : (dtype == DT_F32 ? 4 : 8);
}

static unsigned ew_blocks(long long total)
{
    long long b = (total + 255) / 256;
    if (b > 256 * 32) b = 256 * 32;
    return (unsigned)(b < 1 ? 1 : b);
}

hipError_t launch_bias_add(void* y, const void* bias, int dtype, int bias_f32, int N, int K, int HW, hipStream_t s)
{
    const long long total = (long long)N * K * HW;
    int vec = ew_vector(y, dtype);
    if (HW % vec) vec = 1;
    const dim3 grid(ew_blocks(total / vec)), block(256);
    switch (dtype) {
    case DT_F32:  hipLaunchKernelGGL(bias_add_kernel<DT_F32>, grid, block, 0, s, y, bias, bias_f32, K, HW, total, vec); break;
    case DT_F16:  hipLaunchKernelGGL(bias_add_kernel<DT_F16>, grid, block, 0, s, y, bias, bias_f32, K, HW, total, vec); break;
    case DT_BF16: hipLaunchKernelGGL(bias_add_kernel<DT_BF16>, grid, block, 0, s, y, bias, bias_f32, K, HW, total, vec); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_activation(void* y, int dtype, int act, float alpha, long long total, hipStream_t s)
{
    const int vec = ew_vector(y, dtype);
    const dim3 grid(ew_blocks(total / vec)), block(256);
    switch (dtype) {
    case DT_F32:  hipLaunchKernelGGL(activation_kernel<DT_F32>, grid, block, 0, s, y, act, alpha, total, vec); break;
    case DT_F16:  hipLaunchKernelGGL(activation_kernel<DT_F16>, grid, block, 0, s, y, act, alpha, total, vec); break;
    case DT_BF16: hipLaunchKernelGGL(activation_kernel<DT_BF16>, grid, block, 0, s, y, act, alpha, total, vec); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace cvx
