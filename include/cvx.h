/*
 * cvx.h -- C ABI of the MI355X (gfx950) forward-convolution library.
 *
 * The library computes the forward 2-D convolution of the MIOpen paper (arXiv 1910.00078) with
 * the bias + activation fusion of its Sec. V, on packed NCHW tensors:
 *
 *   input  I[N,C,H,W], filters W[K,C/groups,R,S], output O[N,K,Ho,Wo]        (Fig. 2 tensor roles)
 *   Ho = floor((H + 2*pad_h - dil_h*(R-1) - 1) / stride_h) + 1                (Wo likewise)
 *   O[n,k,p,q] = act( bias[k] + sum_{c,r,s} Iz[n, c0(k)+c, p*stride_h - pad_h + r*dil_h,
 *                                              q*stride_w - pad_w + s*dil_w] * W[k,c,r,s] )
 *   Iz = I inside the image and 0 outside (zero padding, same amount on both sides of an axis);
 *   no filter flip (cross-correlation); c0(k) = (k / (K/groups)) * (C/groups).
 *
 * Conventions common to every call
 *   - Every function returns a cvx_status_t; nothing throws across this boundary; out-parameters
 *     are written only when CVX_OK is returned.
 *   - Handles and descriptors are HOST objects created and destroyed by the caller through the
 *     functions below.  They may be used from one thread at a time.
 *   - All tensor data pointers are DEVICE pointers (HIP global memory of the GPU the handle's
 *     stream belongs to), owned by the caller, packed (no strides), element-aligned.  The library
 *     never allocates, frees or copies device memory and needs no workspace.
 *   - Compute calls only enqueue work on the handle's stream and return; they do not synchronise.
 *     The output buffer must not overlap any input buffer.
 *   - x, w and y must have the same data type.  Arithmetic: products of the stored values,
 *     accumulated in fp32; bias, normalisation and activation applied in fp32; one rounding
 *     (to nearest, ties to even) to the output type at the single store.
 */
#ifndef CVX_H
#define CVX_H

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CVX_OK = 0,
    CVX_ERR_NULL = 1,            /* a required pointer argument is NULL                        */
    CVX_ERR_BAD_PARAM = 2,       /* a dimension / pad / stride / dilation / enum is invalid    */
    CVX_ERR_SHAPE_MISMATCH = 3,  /* descriptors do not describe one consistent convolution     */
    CVX_ERR_UNSUPPORTED = 4,     /* valid request the library has no kernel for                */
    CVX_ERR_ALIGNMENT = 5,       /* a device pointer is not aligned to its element size        */
    CVX_ERR_LAUNCH = 6           /* the HIP runtime refused the launch (see cvx_last_error)    */
} cvx_status_t;

/* Data types the paper lists for convolution (Sec. I); int8 is not provided. */
typedef enum { CVX_F32 = 0, CVX_F16 = 1, CVX_BF16 = 2 } cvx_dtype_t;

/* Activations of the fused epilogue (Sec. V; Table I column "Activations"). */
typedef enum {
    CVX_ACT_IDENTITY = 0,
    CVX_ACT_RELU = 1,            /* max(v, 0)                        */
    CVX_ACT_LEAKY_RELU = 2,      /* v > 0 ? v : alpha * v            */
    CVX_ACT_TANH = 3,
    CVX_ACT_LOGISTIC = 4         /* 1 / (1 + exp(-v))                */
} cvx_act_t;

typedef struct cvx_handle_s*      cvx_handle_t;
typedef struct cvx_tensor_desc_s* cvx_tensor_desc_t;
typedef struct cvx_conv_desc_s*   cvx_conv_desc_t;

/* ---- handle: bound to one HIP stream (Sec. III-D: the handle is created from a HIP stream) ---- */

/* hip_stream is a hipStream_t passed as void*; NULL selects the default stream. */
cvx_status_t cvx_create(cvx_handle_t* out, void* hip_stream);
cvx_status_t cvx_set_stream(cvx_handle_t h, void* hip_stream);
cvx_status_t cvx_get_stream(cvx_handle_t h, void** hip_stream);
cvx_status_t cvx_destroy(cvx_handle_t h);

/* ---- tensor descriptor: packed 4-D, dims (n,c,h,w) (Sec. IV-A: the user constructs the data
 *      structures for the input/output image tensors).  Filters use (K, C/groups, R, S); a bias or
 *      any per-channel vector uses (1, K, 1, 1).  All dims >= 1, fewer than 2^31 elements. ---- */
cvx_status_t cvx_tensor_desc_create(cvx_tensor_desc_t* out);
cvx_status_t cvx_tensor_desc_set_4d(cvx_tensor_desc_t t, cvx_dtype_t dtype, int n, int c, int h, int w);
cvx_status_t cvx_tensor_desc_get_4d(cvx_tensor_desc_t t, cvx_dtype_t* dtype, int* n, int* c, int* h, int* w);
cvx_status_t cvx_tensor_desc_destroy(cvx_tensor_desc_t t);

/* ---- convolution descriptor: padding, striding, dilation (Sec. IV-A) and the group count
 *      (Sec. IV-A "Grouped convolutions"; 1 = ordinary, C = depthwise).  pads >= 0, strides >= 1,
 *      dilations >= 1, groups >= 1.  A new descriptor is pad 0, stride 1, dilation 1, 1 group. ---- */
cvx_status_t cvx_conv_desc_create(cvx_conv_desc_t* out);
cvx_status_t cvx_conv_desc_set_2d(cvx_conv_desc_t c, int pad_h, int pad_w, int stride_h, int stride_w,
                                  int dil_h, int dil_w);
cvx_status_t cvx_conv_desc_set_group_count(cvx_conv_desc_t c, int groups);
cvx_status_t cvx_conv_desc_get_2d(cvx_conv_desc_t c, int* pad_h, int* pad_w, int* stride_h, int* stride_w,
                                  int* dil_h, int* dil_w, int* groups);
cvx_status_t cvx_conv_desc_destroy(cvx_conv_desc_t c);

/* Output dims (N, K, Ho, Wo) by the rule at the top.  CVX_ERR_SHAPE_MISMATCH if x.c != w.c*groups
 * or K % groups != 0; CVX_ERR_BAD_PARAM if the dilated filter does not fit the padded image. */
cvx_status_t cvx_conv_fwd_output_dim(cvx_conv_desc_t c, cvx_tensor_desc_t x, cvx_tensor_desc_t w,
                                     int* n, int* k, int* ho, int* wo);

/* ---- compute ---- */

/* Plain forward convolution (Sec. IV-A): y = conv(x, w); same as the fused call with no bias and
 * the identity activation.  yd must equal cvx_conv_fwd_output_dim(...) and carry x's data type. */
cvx_status_t cvx_conv_fwd(cvx_handle_t h,
                          cvx_tensor_desc_t xd, const void* x,
                          cvx_tensor_desc_t wd, const void* w,
                          cvx_conv_desc_t conv,
                          cvx_tensor_desc_t yd, void* y);

/* Convolution + bias + activation in one kernel (Sec. V, the "CBA" rows of Tables I/II): the
 * intermediate never leaves the chip.  bias may be NULL (then bd is ignored and may be NULL);
 * otherwise bd is (1,K,1,1) with x's data type or CVX_F32.  act_alpha is the leaky-ReLU slope and
 * is ignored by the other activations. */
cvx_status_t cvx_conv_fwd_fused(cvx_handle_t h,
                                cvx_tensor_desc_t xd, const void* x,
                                cvx_tensor_desc_t wd, const void* w,
                                cvx_conv_desc_t conv,
                                cvx_tensor_desc_t bd, const void* bias,
                                cvx_act_t act, float act_alpha,
                                cvx_tensor_desc_t yd, void* y);

/* Convolution + bias + inference-mode spatial batch normalisation + activation (the "CBNA" rows of
 * Tables I/II with the per-channel transform of Sec. IV-B):
 *   v = conv + bias[k];  y = act( scale[k] * (v - mean[k]) / sqrt(var[k] + eps) + shift[k] ).
 * scale, shift, mean, var are device arrays of K fp32 values; bias as in cvx_conv_fwd_fused. */
cvx_status_t cvx_conv_fwd_fused_bn(cvx_handle_t h,
                                   cvx_tensor_desc_t xd, const void* x,
                                   cvx_tensor_desc_t wd, const void* w,
                                   cvx_conv_desc_t conv,
                                   cvx_tensor_desc_t bd, const void* bias,
                                   const float* scale, const float* shift,
                                   const float* mean, const float* var, double eps,
                                   cvx_act_t act, float act_alpha,
                                   cvx_tensor_desc_t yd, void* y);

/* The separate element-wise operators a framework would run without fusion (Sec. V; the unfused
 * side of Fig. 6a): y[n,k,p,q] += bias[k] in place, and y = act(y) in place.  Each reads and writes
 * the whole tensor once, rounding to y's type. */
cvx_status_t cvx_bias_add(cvx_handle_t h, cvx_tensor_desc_t bd, const void* bias,
                          cvx_tensor_desc_t yd, void* y);
cvx_status_t cvx_activation_fwd(cvx_handle_t h, cvx_act_t act, float act_alpha,
                                cvx_tensor_desc_t yd, void* y);

/* What the library would run for this problem, without running it (the find step of Sec. IV-A
 * reduced to its answer: algorithm name and the additional memory it needs -- always 0 here).
 * The answer is for 16-byte-aligned buffers; buffers that are only element-aligned are served by
 * the "direct_*" kernel.  cvx_get_last_kernel names what a compute call actually enqueued.  kernel_name receives a
 * NUL-terminated string of at most name_cap bytes (may be NULL with name_cap 0). */
cvx_status_t cvx_conv_fwd_query(cvx_tensor_desc_t xd, cvx_tensor_desc_t wd, cvx_conv_desc_t conv,
                                cvx_tensor_desc_t yd, char* kernel_name, int name_cap,
                                unsigned long long* workspace_bytes);

/* The kernel the last successful compute call on this handle enqueued ("" before the first). */
cvx_status_t cvx_get_last_kernel(cvx_handle_t h, char* kernel_name, int name_cap);

/* Test and benchmark hooks (no passage of the paper; its auto-tuner, Sec. III-C, plays this role there).
 * cvx_set_kernel_policy: 0 = automatic choice, 1 = generic direct kernel only.
 * cvx_debug_pin_kernel: spec "<kernel name>" or "<igemm kernel name>,<images per tile>,<rows per tile>"
 * makes later compute calls on the handle run exactly that kernel, or fail with
 * CVX_ERR_UNSUPPORTED if it cannot run the problem; NULL or "" removes the pin. */
cvx_status_t cvx_set_kernel_policy(cvx_handle_t h, int policy);
cvx_status_t cvx_debug_pin_kernel(cvx_handle_t h, const char* spec);

const char* cvx_status_string(cvx_status_t s);
const char* cvx_last_error(void);   /* thread-local detail of the last failing call; never NULL */

#ifdef __cplusplus
}
#endif
#endif /* CVX_H */
