// Host side of the C ABI declared in include/cvx.h: handle, descriptors, validation, the
// problem -> kernel selection (the job the MIOpen paper gives its "solvers", Sec. III-A, done here
// by a static table because every kernel is compiled ahead of time), and the launches.
#include "../../include/cvx.h"
#include "cvx_internal.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

// A plan is kept per problem, so that repeated calls (the steady state of training and serving) skip
// the kernel search: the key is every field of the problem that the choice depends on.
struct PlanKey {
    int dtype, N, C, H, W, K, R, S, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w, groups, aligned16, policy, pin_version;
};
struct PlanSlot {
    bool valid;
    PlanKey key;
    cvx::LaunchPlan plan;
};
constexpr int kPlanSlots = 8;

struct cvx_handle_s {
    hipStream_t stream;
    int policy;
    int cus;                       // compute units of the device current when the handle was made
    char pin[96];                  // developer pin, "" = none
    int pin_version;               // bumped whenever the pin changes, so cached plans are not reused across pins
    const char* last_kernel;       // static string: the kernel the last compute call enqueued
    PlanSlot slots[kPlanSlots];
    int next_slot;
};
struct cvx_tensor_desc_s {
    int dtype, n, c, h, w;
    bool set;
};
struct cvx_conv_desc_s {
    int pad_h, pad_w, stride_h, stride_w, dil_h, dil_w, groups;
};

namespace {

thread_local char g_err[512] = "";

cvx_status_t fail(cvx_status_t st, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

bool log_enabled()
{
    static const bool on = [] {
        const char* e = getenv("CVX_LOG");
        return e && *e && *e != '0';
    }();
    return on;
}

int elem_size(int dtype) { return dtype == cvx::DT_F32 ? 4 : 2; }

// Builds the kernel argument block from descriptors, checking everything that can be checked on
// the host.  Data pointers are filled in by the caller.
cvx_status_t build_problem(cvx_tensor_desc_t xd, cvx_tensor_desc_t wd, cvx_conv_desc_t cd,
                           cvx_tensor_desc_t yd, cvx::ConvArgs* out)
{
    if (!xd || !wd || !cd || !yd) return fail(CVX_ERR_NULL, "a descriptor is NULL");
    if (!xd->set || !wd->set || !yd->set) return fail(CVX_ERR_BAD_PARAM, "a tensor descriptor was never set");
    if (xd->dtype != wd->dtype || xd->dtype != yd->dtype)
        return fail(CVX_ERR_UNSUPPORTED, "x, w and y must share one data type (got %d, %d, %d)",
                    xd->dtype, wd->dtype, yd->dtype);
    const int g = cd->groups;
    if (xd->c % g || wd->n % g || xd->c / g != wd->c)
        return fail(CVX_ERR_SHAPE_MISMATCH, "channels: x has %d, filters have %d per group, %d filters, %d groups",
                    xd->c, wd->c, wd->n, g);
    const long long span_h = (long long)xd->h + 2LL * cd->pad_h - (long long)cd->dil_h * (wd->h - 1) - 1;
    const long long span_w = (long long)xd->w + 2LL * cd->pad_w - (long long)cd->dil_w * (wd->w - 1) - 1;
    if (span_h < 0 || span_w < 0)
        return fail(CVX_ERR_BAD_PARAM, "the dilated filter does not fit the padded image (empty output)");
    const long long ho = span_h / cd->stride_h + 1, wo = span_w / cd->stride_w + 1;
    if (yd->n != xd->n || yd->c != wd->n || yd->h != ho || yd->w != wo)
        return fail(CVX_ERR_SHAPE_MISMATCH, "y is (%d,%d,%d,%d) but the convolution produces (%d,%d,%lld,%lld)",
                    yd->n, yd->c, yd->h, yd->w, xd->n, wd->n, ho, wo);
    if ((long long)cd->pad_h + xd->h + cd->pad_h >= (1LL << 30) || (long long)cd->pad_w + xd->w + cd->pad_w >= (1LL << 30))
        return fail(CVX_ERR_BAD_PARAM, "padded extent too large");
    cvx::ConvArgs a;
    memset(&a, 0, sizeof a);
    a.dtype = xd->dtype;
    a.N = xd->n; a.C = xd->c; a.H = xd->h; a.W = xd->w;
    a.K = wd->n; a.R = wd->h; a.S = wd->w;
    a.Ho = (int)ho; a.Wo = (int)wo;
    a.pad_h = cd->pad_h; a.pad_w = cd->pad_w;
    a.stride_h = cd->stride_h; a.stride_w = cd->stride_w;
    a.dil_h = cd->dil_h; a.dil_w = cd->dil_w;
    a.groups = g;
    a.act = cvx::ACT_IDENTITY;
    *out = a;
    return CVX_OK;
}

bool aligned(const void* p, int bytes) { return ((uintptr_t)p % (uintptr_t)bytes) == 0; }

PlanKey make_key(const cvx::ConvArgs& a, bool aligned16, int policy, int pin_version)
{
    PlanKey k;
    memset(&k, 0, sizeof k);                      // padding too: keys are compared bytewise
    k.dtype = a.dtype; k.N = a.N; k.C = a.C; k.H = a.H; k.W = a.W; k.K = a.K; k.R = a.R; k.S = a.S;
    k.pad_h = a.pad_h; k.pad_w = a.pad_w; k.stride_h = a.stride_h; k.stride_w = a.stride_w;
    k.dil_h = a.dil_h; k.dil_w = a.dil_w; k.groups = a.groups;
    k.aligned16 = aligned16 ? 1 : 0; k.policy = policy; k.pin_version = pin_version;
    return k;
}

// The plan for this problem on this handle: from the handle's cache, or made now and cached.
const cvx::LaunchPlan* plan_for(cvx_handle_t h, const cvx::ConvArgs& a)
{
    const bool aligned16 = (((uintptr_t)a.x | (uintptr_t)a.w | (uintptr_t)a.y) & 15) == 0;
    const PlanKey key = make_key(a, aligned16, h->policy, h->pin_version);
    for (int i = 0; i < kPlanSlots; ++i)
        if (h->slots[i].valid && memcmp(&h->slots[i].key, &key, sizeof key) == 0) return &h->slots[i].plan;
    cvx::PlanEnv env;
    env.cus = h->cus;
    env.policy = h->policy;
    env.aligned16 = aligned16;
    env.pin = h->pin[0] ? h->pin : nullptr;
    PlanSlot& slot = h->slots[h->next_slot];
    slot.valid = false;
    if (!cvx::make_plan(a, env, &slot.plan)) return nullptr;
    slot.key = key;
    slot.valid = true;
    h->next_slot = (h->next_slot + 1) % kPlanSlots;
    return &slot.plan;
}

cvx_status_t enqueue(cvx_handle_t h, const cvx::ConvArgs& a)
{
    const cvx::LaunchPlan* p = plan_for(h, a);
    if (!p) return fail(CVX_ERR_UNSUPPORTED, "the pinned kernel \"%s\" cannot run this problem", h->pin);
    if (log_enabled())
        fprintf(stderr, "[cvx] conv_fwd dtype=%d N=%d C=%d H=%d W=%d K=%d R=%d S=%d pad=%d,%d stride=%d,%d dil=%d,%d g=%d -> %s\n",
                a.dtype, a.N, a.C, a.H, a.W, a.K, a.R, a.S, a.pad_h, a.pad_w, a.stride_h, a.stride_w,
                a.dil_h, a.dil_w, a.groups, p->name);
    const hipError_t e = cvx::launch_plan(a, *p, h->stream);
    if (e != hipSuccess) return fail(CVX_ERR_LAUNCH, "%s: %s", p->name, hipGetErrorString(e));
    h->last_kernel = p->name;
    return CVX_OK;
}

cvx_status_t run_conv(cvx_handle_t h, cvx_tensor_desc_t xd, const void* x, cvx_tensor_desc_t wd, const void* w,
                      cvx_conv_desc_t cd, cvx_tensor_desc_t bd, const void* bias,
                      const float* scale, const float* shift, const float* mean, const float* var, double eps,
                      bool with_bn, int act, float alpha, cvx_tensor_desc_t yd, void* y)
{
    if (!h) return fail(CVX_ERR_NULL, "handle is NULL");
    if (!x || !w || !y) return fail(CVX_ERR_NULL, "x, w or y data pointer is NULL");
    cvx::ConvArgs a;
    cvx_status_t st = build_problem(xd, wd, cd, yd, &a);
    if (st != CVX_OK) return st;
    if (act < CVX_ACT_IDENTITY || act > CVX_ACT_LOGISTIC) return fail(CVX_ERR_BAD_PARAM, "unknown activation %d", act);
    if (bias) {
        if (!bd) return fail(CVX_ERR_NULL, "bias given without a descriptor");
        if (!bd->set) return fail(CVX_ERR_BAD_PARAM, "bias descriptor was never set");
        if (bd->n != 1 || bd->c != a.K || bd->h != 1 || bd->w != 1)
            return fail(CVX_ERR_SHAPE_MISMATCH, "bias must be (1,%d,1,1), got (%d,%d,%d,%d)", a.K, bd->n, bd->c, bd->h, bd->w);
        if (bd->dtype != a.dtype && bd->dtype != CVX_F32)
            return fail(CVX_ERR_UNSUPPORTED, "bias must have the data type of x or fp32");
        a.bias_f32 = bd->dtype == CVX_F32;
        if (!aligned(bias, a.bias_f32 ? 4 : elem_size(a.dtype))) return fail(CVX_ERR_ALIGNMENT, "bias pointer misaligned");
    }
    if (with_bn) {
        if (!scale || !shift || !mean || !var) return fail(CVX_ERR_NULL, "a batch-norm array is NULL");
        if (!(eps >= 0.0)) return fail(CVX_ERR_BAD_PARAM, "eps must be >= 0");
        if (!aligned(scale, 4) || !aligned(shift, 4) || !aligned(mean, 4) || !aligned(var, 4))
            return fail(CVX_ERR_ALIGNMENT, "batch-norm arrays must be 4-byte aligned");
        a.bn_scale = scale; a.bn_shift = shift; a.bn_mean = mean; a.bn_var = var; a.bn_eps = (float)eps;
    }
    const int es = elem_size(a.dtype);
    if (!aligned(x, es) || !aligned(w, es) || !aligned(y, es)) return fail(CVX_ERR_ALIGNMENT, "x, w or y is not element-aligned");
    // x, w, bias must not overlap y
    {
        const uintptr_t y0 = (uintptr_t)y, y1 = y0 + (uintptr_t)a.N * a.K * a.Ho * a.Wo * es;
        const uintptr_t x0 = (uintptr_t)x, x1 = x0 + (uintptr_t)a.N * a.C * a.H * a.W * es;
        const uintptr_t w0 = (uintptr_t)w, w1 = w0 + (uintptr_t)a.K * (a.C / a.groups) * a.R * a.S * es;
        if ((x0 < y1 && y0 < x1) || (w0 < y1 && y0 < w1)) return fail(CVX_ERR_BAD_PARAM, "y overlaps an input buffer");
        const auto hits_y = [&](const void* p, size_t bytes) {
            const uintptr_t p0 = (uintptr_t)p;
            return p && p0 < y1 && y0 < p0 + bytes;
        };
        if (hits_y(bias, (size_t)a.K * (a.bias_f32 ? 4 : es)) || hits_y(scale, (size_t)a.K * 4) || hits_y(shift, (size_t)a.K * 4) ||
            hits_y(mean, (size_t)a.K * 4) || hits_y(var, (size_t)a.K * 4))
            return fail(CVX_ERR_BAD_PARAM, "y overlaps the bias or a batch-norm array");
    }
    a.x = x; a.w = w; a.bias = bias; a.y = y;
    a.act = act; a.alpha = alpha;

    return enqueue(h, a);
}

}  // namespace

namespace cvx {

bool make_plan(const ConvArgs& a, const PlanEnv& env, LaunchPlan* out)
{
    if (env.policy == 0) {
        if (env.pin) {
            // the pin names one kernel of one family; nothing else may serve the call
            if (strncmp(env.pin, "pointwise_", 10) == 0) return pointwise_plan(a, env, out);
            if (strncmp(env.pin, "stem_", 5) == 0) return stem_plan(a, env, out);
            if (strncmp(env.pin, "igemm_", 6) == 0) return igemm_plan(a, env, out);
            if (strncmp(env.pin, "tiled_f32_", 10) == 0) return tiled_f32_plan(a, env, out);
            if (strncmp(env.pin, "direct", 6) == 0) return direct_plan(a, env, out);
            return false;
        }
        if (pointwise_plan(a, env, out)) return true;
        if (stem_plan(a, env, out)) return true;
        if (igemm_plan(a, env, out)) return true;
        if (tiled_f32_plan(a, env, out)) return true;
    }
    return direct_plan(a, env, out);
}

hipError_t launch_plan(const ConvArgs& a, const LaunchPlan& p, hipStream_t s)
{
    switch (p.id) {
    case KID_IGEMM:     return igemm_launch(a, p, s);
    case KID_STEM:      return stem_launch(a, p, s);
    case KID_POINTWISE: return pointwise_launch(a, p, s);
    case KID_TILED_F32: return tiled_f32_launch(a, p, s);
    default:            return direct_launch(a, p, s);
    }
}

}  // namespace cvx

extern "C" {

cvx_status_t cvx_create(cvx_handle_t* out, void* hip_stream)
{
    if (!out) return fail(CVX_ERR_NULL, "out is NULL");
    cvx_handle_s* h = new (std::nothrow) cvx_handle_s;
    if (!h) return fail(CVX_ERR_BAD_PARAM, "out of host memory");
    memset(h, 0, sizeof *h);
    h->stream = (hipStream_t)hip_stream;
    h->last_kernel = "";
    // With a device present: its compute-unit count, and the kernels' LDS limits raised now rather than
    // inside the first compute call (which may be under stream capture).  Without one (host-only use of
    // the descriptor and query calls) the MI355X count stands in.
    h->cus = 256;
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) {
        h->cus = n;
        (void)cvx::igemm_prepare();
        (void)cvx::stem_prepare();
        (void)cvx::pointwise_prepare();
        (void)cvx::tiled_f32_prepare();
    }
    (void)hipGetLastError();
    *out = h;
    return CVX_OK;
}

cvx_status_t cvx_get_last_kernel(cvx_handle_t h, char* kernel_name, int name_cap)
{
    if (!h || !kernel_name) return fail(CVX_ERR_NULL, "NULL argument");
    if (name_cap < 1) return fail(CVX_ERR_BAD_PARAM, "bad name buffer");
    strncpy(kernel_name, h->last_kernel, (size_t)name_cap - 1);
    kernel_name[name_cap - 1] = '\0';
    return CVX_OK;
}

cvx_status_t cvx_debug_pin_kernel(cvx_handle_t h, const char* spec)
{
    if (!h) return fail(CVX_ERR_NULL, "handle is NULL");
    if (spec && strlen(spec) >= sizeof h->pin) return fail(CVX_ERR_BAD_PARAM, "pin too long");
    snprintf(h->pin, sizeof h->pin, "%s", spec ? spec : "");
    ++h->pin_version;
    return CVX_OK;
}

cvx_status_t cvx_set_stream(cvx_handle_t h, void* hip_stream)
{
    if (!h) return fail(CVX_ERR_NULL, "handle is NULL");
    h->stream = (hipStream_t)hip_stream;
    return CVX_OK;
}

cvx_status_t cvx_get_stream(cvx_handle_t h, void** hip_stream)
{
    if (!h || !hip_stream) return fail(CVX_ERR_NULL, "NULL argument");
    *hip_stream = (void*)h->stream;
    return CVX_OK;
}

cvx_status_t cvx_destroy(cvx_handle_t h)
{
    if (!h) return fail(CVX_ERR_NULL, "handle is NULL");
    delete h;
    return CVX_OK;
}

cvx_status_t cvx_set_kernel_policy(cvx_handle_t h, int policy)
{
    if (!h) return fail(CVX_ERR_NULL, "handle is NULL");
    if (policy < 0 || policy > 1) return fail(CVX_ERR_BAD_PARAM, "policy must be 0 or 1");
    h->policy = policy;
    return CVX_OK;
}

cvx_status_t cvx_tensor_desc_create(cvx_tensor_desc_t* out)
{
    if (!out) return fail(CVX_ERR_NULL, "out is NULL");
    cvx_tensor_desc_s* t = new (std::nothrow) cvx_tensor_desc_s;
    if (!t) return fail(CVX_ERR_BAD_PARAM, "out of host memory");
    memset(t, 0, sizeof *t);
    *out = t;
    return CVX_OK;
}

cvx_status_t cvx_tensor_desc_set_4d(cvx_tensor_desc_t t, cvx_dtype_t dtype, int n, int c, int h, int w)
{
    if (!t) return fail(CVX_ERR_NULL, "descriptor is NULL");
    if (dtype != CVX_F32 && dtype != CVX_F16 && dtype != CVX_BF16) return fail(CVX_ERR_BAD_PARAM, "unknown data type %d", (int)dtype);
    if (n < 1 || c < 1 || h < 1 || w < 1) return fail(CVX_ERR_BAD_PARAM, "dims must be >= 1 (got %d,%d,%d,%d)", n, c, h, w);
    if ((long long)n * c * h * w >= (1LL << 31)) return fail(CVX_ERR_BAD_PARAM, "tensor has 2^31 or more elements");
    t->dtype = (int)dtype; t->n = n; t->c = c; t->h = h; t->w = w; t->set = true;
    return CVX_OK;
}

cvx_status_t cvx_tensor_desc_get_4d(cvx_tensor_desc_t t, cvx_dtype_t* dtype, int* n, int* c, int* h, int* w)
{
    if (!t || !dtype || !n || !c || !h || !w) return fail(CVX_ERR_NULL, "NULL argument");
    if (!t->set) return fail(CVX_ERR_BAD_PARAM, "descriptor was never set");
    *dtype = (cvx_dtype_t)t->dtype; *n = t->n; *c = t->c; *h = t->h; *w = t->w;
    return CVX_OK;
}

cvx_status_t cvx_tensor_desc_destroy(cvx_tensor_desc_t t)
{
    if (!t) return fail(CVX_ERR_NULL, "descriptor is NULL");
    delete t;
    return CVX_OK;
}

cvx_status_t cvx_conv_desc_create(cvx_conv_desc_t* out)
{
    if (!out) return fail(CVX_ERR_NULL, "out is NULL");
    cvx_conv_desc_s* c = new (std::nothrow) cvx_conv_desc_s;
    if (!c) return fail(CVX_ERR_BAD_PARAM, "out of host memory");
    c->pad_h = c->pad_w = 0;
    c->stride_h = c->stride_w = c->dil_h = c->dil_w = c->groups = 1;
    *out = c;
    return CVX_OK;
}

cvx_status_t cvx_conv_desc_set_2d(cvx_conv_desc_t c, int pad_h, int pad_w, int stride_h, int stride_w, int dil_h, int dil_w)
{
    if (!c) return fail(CVX_ERR_NULL, "descriptor is NULL");
    if (pad_h < 0 || pad_w < 0) return fail(CVX_ERR_BAD_PARAM, "padding must be >= 0");
    if (stride_h < 1 || stride_w < 1) return fail(CVX_ERR_BAD_PARAM, "stride must be >= 1");
    if (dil_h < 1 || dil_w < 1) return fail(CVX_ERR_BAD_PARAM, "dilation must be >= 1");
    c->pad_h = pad_h; c->pad_w = pad_w; c->stride_h = stride_h; c->stride_w = stride_w; c->dil_h = dil_h; c->dil_w = dil_w;
    return CVX_OK;
}

cvx_status_t cvx_conv_desc_set_group_count(cvx_conv_desc_t c, int groups)
{
    if (!c) return fail(CVX_ERR_NULL, "descriptor is NULL");
    if (groups < 1) return fail(CVX_ERR_BAD_PARAM, "group count must be >= 1");
    c->groups = groups;
    return CVX_OK;
}

cvx_status_t cvx_conv_desc_get_2d(cvx_conv_desc_t c, int* pad_h, int* pad_w, int* stride_h, int* stride_w,
                                  int* dil_h, int* dil_w, int* groups)
{
    if (!c || !pad_h || !pad_w || !stride_h || !stride_w || !dil_h || !dil_w || !groups) return fail(CVX_ERR_NULL, "NULL argument");
    *pad_h = c->pad_h; *pad_w = c->pad_w; *stride_h = c->stride_h; *stride_w = c->stride_w;
    *dil_h = c->dil_h; *dil_w = c->dil_w; *groups = c->groups;
    return CVX_OK;
}

cvx_status_t cvx_conv_desc_destroy(cvx_conv_desc_t c)
{
    if (!c) return fail(CVX_ERR_NULL, "descriptor is NULL");
    delete c;
    return CVX_OK;
}

cvx_status_t cvx_conv_fwd_output_dim(cvx_conv_desc_t c, cvx_tensor_desc_t x, cvx_tensor_desc_t w,
                                     int* n, int* k, int* ho, int* wo)
{
    if (!c || !x || !w || !n || !k || !ho || !wo) return fail(CVX_ERR_NULL, "NULL argument");
    if (!x->set || !w->set) return fail(CVX_ERR_BAD_PARAM, "a tensor descriptor was never set");
    if (x->c % c->groups || w->n % c->groups || x->c / c->groups != w->c)
        return fail(CVX_ERR_SHAPE_MISMATCH, "channels: x has %d, filters have %d per group, %d filters, %d groups",
                    x->c, w->c, w->n, c->groups);
    const long long span_h = (long long)x->h + 2LL * c->pad_h - (long long)c->dil_h * (w->h - 1) - 1;
    const long long span_w = (long long)x->w + 2LL * c->pad_w - (long long)c->dil_w * (w->w - 1) - 1;
    if (span_h < 0 || span_w < 0) return fail(CVX_ERR_BAD_PARAM, "the dilated filter does not fit the padded image (empty output)");
    const long long oh = span_h / c->stride_h + 1, ow = span_w / c->stride_w + 1;
    if ((long long)x->n * w->n * oh * ow >= (1LL << 31)) return fail(CVX_ERR_BAD_PARAM, "output has 2^31 or more elements");
    *n = x->n; *k = w->n; *ho = (int)oh; *wo = (int)ow;
    return CVX_OK;
}

cvx_status_t cvx_conv_fwd(cvx_handle_t h, cvx_tensor_desc_t xd, const void* x, cvx_tensor_desc_t wd, const void* w,
                          cvx_conv_desc_t conv, cvx_tensor_desc_t yd, void* y)
{
    return run_conv(h, xd, x, wd, w, conv, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0.0, false,
                    CVX_ACT_IDENTITY, 0.0f, yd, y);
}

cvx_status_t cvx_conv_fwd_fused(cvx_handle_t h, cvx_tensor_desc_t xd, const void* x, cvx_tensor_desc_t wd, const void* w,
                                cvx_conv_desc_t conv, cvx_tensor_desc_t bd, const void* bias,
                                cvx_act_t act, float act_alpha, cvx_tensor_desc_t yd, void* y)
{
    return run_conv(h, xd, x, wd, w, conv, bd, bias, nullptr, nullptr, nullptr, nullptr, 0.0, false,
                    (int)act, act_alpha, yd, y);
}

cvx_status_t cvx_conv_fwd_fused_bn(cvx_handle_t h, cvx_tensor_desc_t xd, const void* x, cvx_tensor_desc_t wd, const void* w,
                                   cvx_conv_desc_t conv, cvx_tensor_desc_t bd, const void* bias,
                                   const float* scale, const float* shift, const float* mean, const float* var, double eps,
                                   cvx_act_t act, float act_alpha, cvx_tensor_desc_t yd, void* y)
{
    return run_conv(h, xd, x, wd, w, conv, bd, bias, scale, shift, mean, var, eps, true, (int)act, act_alpha, yd, y);
}

cvx_status_t cvx_bias_add(cvx_handle_t h, cvx_tensor_desc_t bd, const void* bias, cvx_tensor_desc_t yd, void* y)
{
    if (!h || !bd || !yd || !bias || !y) return fail(CVX_ERR_NULL, "NULL argument");
    if (!bd->set || !yd->set) return fail(CVX_ERR_BAD_PARAM, "a tensor descriptor was never set");
    if (bd->n != 1 || bd->c != yd->c || bd->h != 1 || bd->w != 1)
        return fail(CVX_ERR_SHAPE_MISMATCH, "bias must be (1,%d,1,1)", yd->c);
    if (bd->dtype != yd->dtype && bd->dtype != CVX_F32) return fail(CVX_ERR_UNSUPPORTED, "bias must have y's data type or fp32");
    const int bias_f32 = bd->dtype == CVX_F32;
    if (!aligned(y, elem_size(yd->dtype)) || !aligned(bias, bias_f32 ? 4 : elem_size(yd->dtype)))
        return fail(CVX_ERR_ALIGNMENT, "pointer misaligned");
    hipError_t e = cvx::launch_bias_add(y, bias, yd->dtype, bias_f32, yd->n, yd->c, yd->h * yd->w, h->stream);
    if (e != hipSuccess) return fail(CVX_ERR_LAUNCH, "bias_add: %s", hipGetErrorString(e));
    return CVX_OK;
}

cvx_status_t cvx_activation_fwd(cvx_handle_t h, cvx_act_t act, float act_alpha, cvx_tensor_desc_t yd, void* y)
{
    if (!h || !yd || !y) return fail(CVX_ERR_NULL, "NULL argument");
    if (!yd->set) return fail(CVX_ERR_BAD_PARAM, "tensor descriptor was never set");
    if (act < CVX_ACT_IDENTITY || act > CVX_ACT_LOGISTIC) return fail(CVX_ERR_BAD_PARAM, "unknown activation %d", (int)act);
    if (!aligned(y, elem_size(yd->dtype))) return fail(CVX_ERR_ALIGNMENT, "pointer misaligned");
    hipError_t e = cvx::launch_activation(y, yd->dtype, (int)act, act_alpha, (long long)yd->n * yd->c * yd->h * yd->w, h->stream);
    if (e != hipSuccess) return fail(CVX_ERR_LAUNCH, "activation: %s", hipGetErrorString(e));
    return CVX_OK;
}

cvx_status_t cvx_conv_fwd_query(cvx_tensor_desc_t xd, cvx_tensor_desc_t wd, cvx_conv_desc_t conv, cvx_tensor_desc_t yd,
                                char* kernel_name, int name_cap, unsigned long long* workspace_bytes)
{
    cvx::ConvArgs a;
    cvx_status_t st = build_problem(xd, wd, conv, yd, &a);
    if (st != CVX_OK) return st;
    if (name_cap < 0 || (name_cap > 0 && !kernel_name)) return fail(CVX_ERR_BAD_PARAM, "bad name buffer");
    // No pointers here: the answer is for 16-byte-aligned buffers (what device allocators give) and the
    // automatic policy.
    cvx::PlanEnv env;
    env.cus = 256;
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) env.cus = n;
    (void)hipGetLastError();
    env.policy = 0;
    env.aligned16 = true;
    env.pin = nullptr;
    cvx::LaunchPlan plan;
    cvx::make_plan(a, env, &plan);
    if (kernel_name && name_cap > 0) {
        strncpy(kernel_name, plan.name, (size_t)name_cap - 1);
        kernel_name[name_cap - 1] = '\0';
    }
    if (workspace_bytes) *workspace_bytes = 0ull;      // no kernel of this library uses a workspace
    return CVX_OK;
}

const char* cvx_status_string(cvx_status_t s)
{
    switch (s) {
    case CVX_OK: return "CVX_OK";
    case CVX_ERR_NULL: return "CVX_ERR_NULL";
    case CVX_ERR_BAD_PARAM: return "CVX_ERR_BAD_PARAM";
    case CVX_ERR_SHAPE_MISMATCH: return "CVX_ERR_SHAPE_MISMATCH";
    case CVX_ERR_UNSUPPORTED: return "CVX_ERR_UNSUPPORTED";
    case CVX_ERR_ALIGNMENT: return "CVX_ERR_ALIGNMENT";
    case CVX_ERR_LAUNCH: return "CVX_ERR_LAUNCH";
    default: return "CVX_ERR_UNKNOWN";
    }
}

const char* cvx_last_error(void) { return g_err; }

}  // extern "C"
