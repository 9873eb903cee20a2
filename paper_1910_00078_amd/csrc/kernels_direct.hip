// Generic direct forward convolution: one thread per output element, any filter size, padding,
// stride, dilation and group count, all three data types, fp32 accumulation, fused epilogue.
// This is the correctness net behind the specialised kernels (the "direct" family of Sec. IV-A of
// the MIOpen paper in its plainest form), plus the separate bias / activation operators that the
// unfused path of Sec. V uses.
#include "cvx_device.h"

namespace cvx {

template <int DT>
__global__ void __launch_bounds__(256) direct_conv_kernel(ConvArgs a)
{
    const long long total = (long long)a.N * a.K * a.Ho * a.Wo;
    const int cg = a.C / a.groups;
    const int kg = a.K / a.groups;
    const bool has_bn = a.bn_scale != nullptr;
    for (long long o = (long long)blockIdx.x * blockDim.x + threadIdx.x; o < total;
         o += (long long)gridDim.x * blockDim.x) {
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
        for (int c = 0; c < cg; ++c) {
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
        const ChannelAffine ca = channel_affine<DT>(a, k);
        Elem<DT>::store(a.y, (size_t)o, finish(acc, ca, has_bn, a.act, a.alpha));
    }
}

hipError_t launch_direct(const ConvArgs& a, hipStream_t s)
{
    const long long total = (long long)a.N * a.K * a.Ho * a.Wo;
    long long blocks = (total + 255) / 256;
    if (blocks > (1 << 20)) blocks = 1 << 20;           // grid-stride loop covers the rest
    const dim3 grid((unsigned)blocks), block(256);
    switch (a.dtype) {
    case DT_F32:  hipLaunchKernelGGL(direct_conv_kernel<DT_F32>, grid, block, 0, s, a); break;
    case DT_F16:  hipLaunchKernelGGL(direct_conv_kernel<DT_F16>, grid, block, 0, s, a); break;
    case DT_BF16: hipLaunchKernelGGL(direct_conv_kernel<DT_BF16>, grid, block, 0, s, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ---- unfused element-wise operators --------------------------------------------------------------
template <int DT>
__global__ void __launch_bounds__(256) bias_add_kernel(void* y, const void* bias, int bias_f32,
                                                        int K, int HW, long long total)
{
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const int k = (int)((i / HW) % K);
        const float b = bias_f32 ? ((const float*)bias)[k] : Elem<DT>::load(bias, k);
        Elem<DT>::store(y, (size_t)i, Elem<DT>::load(y, (size_t)i) + b);
    }
}

template <int DT>
__global__ void __launch_bounds__(256) activation_kernel(void* y, int act, float alpha, long long total)
{
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x)
        Elem<DT>::store(y, (size_t)i, activate(Elem<DT>::load(y, (size_t)i), act, alpha));
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
    const dim3 grid(ew_blocks(total)), block(256);
    switch (dtype) {
    case DT_F32:  hipLaunchKernelGGL(bias_add_kernel<DT_F32>, grid, block, 0, s, y, bias, bias_f32, K, HW, total); break;
    case DT_F16:  hipLaunchKernelGGL(bias_add_kernel<DT_F16>, grid, block, 0, s, y, bias, bias_f32, K, HW, total); break;
    case DT_BF16: hipLaunchKernelGGL(bias_add_kernel<DT_BF16>, grid, block, 0, s, y, bias, bias_f32, K, HW, total); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_activation(void* y, int dtype, int act, float alpha, long long total, hipStream_t s)
{
    const dim3 grid(ew_blocks(total)), block(256);
    switch (dtype) {
    case DT_F32:  hipLaunchKernelGGL(activation_kernel<DT_F32>, grid, block, 0, s, y, act, alpha, total); break;
    case DT_F16:  hipLaunchKernelGGL(activation_kernel<DT_F16>, grid, block, 0, s, y, act, alpha, total); break;
    case DT_BF16: hipLaunchKernelGGL(activation_kernel<DT_BF16>, grid, block, 0, s, y, act, alpha, total); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace cvx
