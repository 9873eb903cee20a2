// Device-side helpers shared by the kernels: storage-type conversion and the fused epilogue
// (bias, optional inference batch-norm, activation -- Sec. V and Tables I/II of the MIOpen paper).
#pragma once
#include "cvx_internal.h"

namespace cvx {

typedef _Float16 half_t;

// ---- storage <-> fp32 ------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Round to nearest, ties to even; NaN stays NaN (quiet).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ uint16_t f32_to_f16_bits(float f)
{
    half_t h = (half_t)f;                       // v_cvt_f16_f32: round to nearest even
    return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ float f16_bits_to_f32(uint16_t b) { return (float)__builtin_bit_cast(half_t, b); }

template <int DT> struct Elem;
template <> struct Elem<DT_F32> {
    typedef float type;
    static __device__ __forceinline__ float load(const void* p, size_t i) { return ((const float*)p)[i]; }
    static __device__ __forceinline__ void store(void* p, size_t i, float v) { ((float*)p)[i] = v; }
};
template <> struct Elem<DT_F16> {
    typedef uint16_t type;
    static __device__ __forceinline__ float load(const void* p, size_t i) { return f16_bits_to_f32(((const uint16_t*)p)[i]); }
    static __device__ __forceinline__ void store(void* p, size_t i, float v) { ((uint16_t*)p)[i] = f32_to_f16_bits(v); }
};
template <> struct Elem<DT_BF16> {
    typedef uint16_t type;
    static __device__ __forceinline__ float load(const void* p, size_t i) { return bf16_bits_to_f32(((const uint16_t*)p)[i]); }
    static __device__ __forceinline__ void store(void* p, size_t i, float v) { ((uint16_t*)p)[i] = f32_to_bf16_bits(v); }
};

// 16-bit storage conversion selected at compile time (DT_F16 or DT_BF16).
template <int DT> __device__ __forceinline__ uint16_t f32_to_bits16(float v)
{
    return DT == DT_BF16 ? f32_to_bf16_bits(v) : f32_to_f16_bits(v);
}
template <int DT> __device__ __forceinline__ float bits16_to_f32(uint16_t b)
{
    return DT == DT_BF16 ? bf16_bits_to_f32(b) : f16_bits_to_f32(b);
}

// ---- epilogue ----------------------------------------------------------------------------------
__device__ __forceinline__ float activate(float v, int act, float alpha)
{
    switch (act) {
    case ACT_RELU:       return fmaxf(v, 0.0f);
    case ACT_LEAKY_RELU: return v > 0.0f ? v : alpha * v;
    case ACT_TANH:       return tanhf(v);
    case ACT_LOGISTIC:   return 1.0f / (1.0f + expf(-v));
    default:             return v;
    }
}

// Per-output-channel affine form of the epilogue: y = act(acc * mul + add), with
//   no batch-norm:  mul = 1,                          add = bias
//   batch-norm:     mul = scale / sqrt(var + eps),    add = (bias - mean) * mul + shift
struct ChannelAffine {
    float mul, add;
};

template <int DT>
__device__ __forceinline__ ChannelAffine channel_affine(const ConvArgs& a, int k)
{
    float b = 0.0f;
    if (a.bias) b = a.bias_f32 ? ((const float*)a.bias)[k] : Elem<DT>::load(a.bias, k);
    ChannelAffine r;
    if (a.bn_scale) {
        const float m = a.bn_scale[k] / sqrtf(a.bn_var[k] + a.bn_eps);
        r.mul = m;
        r.add = (b - a.bn_mean[k]) * m + a.bn_shift[k];
    } else {
        r.mul = 1.0f;
        r.add = b;
    }
    return r;
}

__device__ __forceinline__ float finish(float acc, const ChannelAffine& ca, bool has_bn, int act, float alpha)
{
    const float v = has_bn ? fmaf(acc, ca.mul, ca.add) : acc + ca.add;
    return activate(v, act, alpha);
}

// The bias + ReLU (or identity) epilogue on values already rounded to bf16 / fp16 and packed two to
// a dword.  Both formats are sign-magnitude, so as signed 16-bit integers the negative values are
// exactly the negative integers: max(v, 0) is ReLU, max(v, -32768) the identity, one v_pk_max_i16 for
// two values.  Rounding before the ReLU gives the same result as after it (rounding keeps the sign).
typedef short s16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t packed_floor(bool relu)
{
    return relu ? 0u : 0x80008000u;
}
__device__ __forceinline__ uint32_t max_packed(uint32_t v, uint32_t floor2)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2_t, v), __builtin_bit_cast(s16x2_t, floor2)));
}

// ---- vector types, the 16-bit matrix instruction and the packed output conversion, shared by the MFMA kernels
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_a2 __attribute__((ext_vector_type(4), aligned(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// v_mfma_f32_32x32x16 (bf16 or f16 in, fp32 accumulate): a and b hold a lane's 8 consecutive reduction elements.
template <int DT>
__device__ __forceinline__ f32x16 mfma_32x32x16(u32x4 a, u32x4 b, f32x16 c)
{
    if constexpr (DT == DT_BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Two fp32 values -> one dword of two bf16 / fp16 values (lo in bits 0..15), round to nearest even
// in hardware (v_cvt_pk_bf16_f32 / v_cvt_pk_f16_f32).
template <int DT>
__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    if constexpr (DT == DT_BF16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    else return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

// Fetches the first BYTES bytes of the kernel-argument segment with a few wide scalar loads that
// are all in flight together, and waits for them once.  The compiler otherwise fetches arguments
// where they are first needed, and a kernel prologue that decodes its tile from several of them
// then pays the (cold) argument-memory latency several times in a row; after this call every later
// argument fetch hits the scalar cache.  BYTES must not exceed the size of the explicit arguments.
template <int BYTES>
__device__ __forceinline__ void warm_kernel_arguments()
{
    typedef uint32_t u32x16_s __attribute__((ext_vector_type(16)));
    typedef const __attribute__((address_space(4))) uint32_t* karg_ptr;
    typedef const __attribute__((address_space(4))) u32x16_s* karg16_ptr;
    const karg_ptr ka = (karg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
    // one 64-byte load per cache line of the arguments; a single asm statement takes all results, so
    // the loads are issued back to back and waited for together
    constexpr int N16 = BYTES / 64;
    static_assert(N16 >= 1 && N16 <= 5, "argument block size not covered");
    const karg16_ptr k16 = (karg16_ptr)ka;
    const uint32_t last = ka[BYTES / 4 - 1];      // the line holding the tail of the arguments
    if constexpr (N16 == 1) asm volatile("" ::"s"(k16[0]), "s"(last));
    if constexpr (N16 == 2) asm volatile("" ::"s"(k16[0]), "s"(k16[1]), "s"(last));
    if constexpr (N16 == 3) asm volatile("" ::"s"(k16[0]), "s"(k16[1]), "s"(k16[2]), "s"(last));
    if constexpr (N16 == 4) asm volatile("" ::"s"(k16[0]), "s"(k16[1]), "s"(k16[2]), "s"(k16[3]), "s"(last));
    if constexpr (N16 == 5) asm volatile("" ::"s"(k16[0]), "s"(k16[1]), "s"(k16[2]), "s"(k16[3]), "s"(k16[4]), "s"(last));
}

// Developer facility, compiled out unless CVX_PHASE_TRACE is defined: thread 0 of every block
// records wall-clock timestamps (100 MHz) at phase boundaries into a caller-provided buffer of
// 32 slots per block (16 wall-clock stamps, then 16 shader-clock stamps).
#ifdef CVX_PHASE_TRACE
static __device__ unsigned long long* g_phase_trace = nullptr;   // one per translation unit
#define CVX_TRACE_MARK(slot) CVX_TRACE_MARK_T(slot, 0)
#define CVX_TRACE_MARK_T(slot, t)                                                                 \
    do {                                                                                          \
        if (threadIdx.x == (t) && g_phase_trace) {                                                  \
            g_phase_trace[(size_t)blockIdx.x * 32 + (slot)] = wall_clock64();                     \
            g_phase_trace[(size_t)blockIdx.x * 32 + 16 + (slot)] = clock64();                     \
        }                                                                                         \
    } while (0)
#else
#define CVX_TRACE_MARK(slot) do { } while (0)
#define CVX_TRACE_MARK_T(slot, t) do { } while (0)
#endif


}  // namespace cvx
