// Forward convolution in fp32 on the fp32 matrix instruction (v_mfma_f32_32x32x2_f32) for gfx950,
// with the bias / batch-norm / activation epilogue of Sec. V of the MIOpen paper applied to the
// accumulators before the single store.  Any filter size, padding, stride, dilation and group
// count; the structure is Fig. 2's: blockwise slices of the input and the filters into LDS, threadwise
// fragments from LDS into registers, accumulation in registers over (channel chunk, Y, X), one copy out.
//
//   GEMM view      D[pix][k] = sum_{c, tap} X[pix @ tap][c] * W[k][c][tap]
//   MFMA           32 pixels x 32 filters x 2 reduction elements per instruction; the two reduction
//                  elements are two consecutive channels at one filter tap.  A lane supplies ONE fp32
//                  of each operand, so -- unlike the 16-bit kernels, whose lanes want 8 consecutive
//                  channels -- nothing has to be transposed: pixels stay contiguous as in NCHW.
//   Input in LDS   [channel][image][patch row][WP] as in memory, with the pad columns as zeros.
//   Filters in LDS [filter][channel * taps + tap] as in memory (KCRS), pitch odd so that the 32 lanes
//                  of a fragment read (32 filters, one reduction element) fall on 32 banks.
//   Pipeline       two LDS buffers; the next chunk's global loads are in flight (in registers) while
//                  the current one is multiplied; one barrier per chunk.
//   Price          the fp32 matrix pipe peaks where the fp32 vector pipe does (157.3 TFLOP/s), but
//                  needs two LDS dwords per 4096 FLOP instead of two per 2.
#include "cvx_device.h"

#include <cstring>

namespace cvx {

namespace tf32 {

struct Geom {
    int NB, TH, PH, WP;          // images and output rows per pixel tile; input rows a tile needs; LDS row pitch (floats)
    int plane;                   // floats per channel in LDS: NB * PH * WP, padded to 32 (mod 64)
    int row_blocks, img_blocks, k_blocks, kb_per_group, cg, kg;
    int n_stages;                // ceil(cg / CC)
    int x_elems, w_elems;        // floats staged per chunk: CC * NB * PH * W and KT * CC * taps
    int wpitch;                  // floats per filter row in LDS: CC * taps, made odd
    int xfloats, wfloats;        // LDS floats per buffer for input and filters
    int xorg;                    // LDS rows start with xorg unused floats, so that image column 0 sits on a 16-byte boundary (vector staging)
    int x_units, w_units;        // 16-byte pieces staged per chunk (vector staging)
    int vec;                     // 1: the vector-staging kernel runs
};


constexpr int THREADS = 256;
constexpr int XE = 16;           // input elements a thread stages per chunk, at most
constexpr int WE = 24;           // filter elements a thread stages per chunk, at most
constexpr int XV = 4, WV = 6;    // the same in 16-byte pieces (vector staging)

// WM x WN waves, each TM x TN tiles of 32 pixels x 32 filters; CC channels per chunk; TAPS = R * S
// compiled in (the multiply loop is then fully unrolled, with the next step's fragments read while the
// current step multiplies), or 0 for any filter size.
// VEC: the chunk is staged in 16-byte pieces (image rows and filter rows that are multiples of four floats on
// 16-byte boundaries, whole channel chunks): a quarter of the load and LDS-write instructions and half the
// registers of the element-wise staging, which serves every other shape.
template <int WM, int WN, int TM, int TN, int CC, int TAPS, bool VEC>
__global__ void __launch_bounds__(THREADS) tiled_f32_kernel(ConvArgs a, Geom g)
{
    static_assert(WM * WN * 64 == THREADS && CC % 2 == 0 && CC <= 16 && XE <= 16 && WE <= 32, "four waves, channel pairs, 4-bit channel indices");
    constexpr int KT = WN * TN * 32;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    warm_kernel_arguments<sizeof(ConvArgs) + sizeof(Geom)>();
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int taps = TAPS > 0 ? TAPS : a.R * a.S;
    const int HW = a.H * a.W, HoWo = a.Ho * a.Wo;

    // ---- which tile (filter block fastest: neighbours share an input tile)
    const int lid = blockIdx.x;
    const int pb = lid / g.k_blocks, kb = lid - pb * g.k_blocks;
    const int ib = pb / g.row_blocks, rb = pb - ib * g.row_blocks;
    const int grp = kb / g.kb_per_group;
    const int k0 = grp * g.kg + (kb - grp * g.kb_per_group) * KT;
    const int k_end = (grp + 1) * g.kg;
    const int c_first = grp * g.cg;
    const int n0 = ib * g.NB, p0 = rb * g.TH;
    const int rows = min(g.TH, a.Ho - p0);
    const int nimg = min(g.NB, a.N - n0);
    const int ppi = rows * a.Wo;                       // output pixels per image in this tile
    const int npix = nimg * ppi;
    const int h_lo = p0 * a.stride_h - a.pad_h;        // first input row of the patch (may be < 0)

    const float* __restrict__ xg = (const float*)a.x;
    const float* __restrict__ wg = (const float*)a.w;
    const int buf_floats = g.xfloats + g.wfloats;

    // ---- what this thread stages per chunk: fixed positions, only the channel base moves
    constexpr int NXE = VEC ? 1 : XE, NWE = VEC ? 1 : WE, NXV = VEC ? XV : 1, NWV = VEC ? WV : 1;
    int x_src[NXE], x_dst[NXE];                        // global offset inside a channel chunk (-1: zero), LDS float offset (-1: none)
    unsigned long long x_ch = 0ull;                    // 4 bits per element: its channel inside the chunk
    int w_src[NWE], w_dst[NWE];
    unsigned long long w_ch[2] = {0ull, 0ull};
    int xv_src[NXV], xv_dst[NXV], wv_src[NWV], wv_dst[NWV];   // vector staging: -1 = nothing to fetch (LDS keeps its zeros)
    if constexpr (!VEC) {
        const int per_c = g.NB * g.PH * a.W;
#pragma unroll
        for (int i = 0; i < XE; ++i) {
            const int e = tid + i * THREADS;
            x_src[i] = -1;
            x_dst[i] = -1;
            if (e < g.x_elems) {
                const int c = e / per_c, r1 = e - c * per_c;
                const int img = r1 / (g.PH * a.W), r2 = r1 - img * (g.PH * a.W);
                const int row = r2 / a.W, col = r2 - row * a.W;
                const int h = h_lo + row;
                x_dst[i] = c * g.plane + (img * g.PH + row) * g.WP + col + a.pad_w;
                x_ch |= (unsigned long long)c << (4 * i);
                if (img < nimg && h >= 0 && h < a.H) x_src[i] = ((img * a.C + c) * a.H + h) * a.W + col;
            }
        }
        const int per_k = CC * taps;
#pragma unroll
        for (int i = 0; i < WE; ++i) {
            const int e = tid + i * THREADS;
            w_src[i] = -1;
            w_dst[i] = -1;
            if (e < g.w_elems) {
                const int k = e / per_k, j = e - k * per_k;
                w_dst[i] = k * g.wpitch + j;
                w_ch[i >> 4] |= (unsigned long long)(j / taps) << (4 * (i & 15));
                if (k0 + k < k_end) w_src[i] = k * g.cg * taps + j;      // j = c * taps + tap, contiguous in memory
            }
        }
    } else {
        const int w4 = a.W >> 2, per_c = g.NB * g.PH * w4;
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            const int u = tid + i * THREADS;
            xv_src[i] = xv_dst[i] = -1;
            if (u < g.x_units) {
                const int c = u / per_c, r1 = u - c * per_c;
                const int img = r1 / (g.PH * w4), r2 = r1 - img * (g.PH * w4);
                const int row = r2 / w4, col = 4 * (r2 - row * w4);
                const int h = h_lo + row;
                if (img < nimg && h >= 0 && h < a.H) {
                    xv_src[i] = ((img * a.C + c) * a.H + h) * a.W + col;
                    xv_dst[i] = c * g.plane + (img * g.PH + row) * g.WP + g.xorg + a.pad_w + col;
                }
            }
        }
        const int per_k = (CC * taps) >> 2;
#pragma unroll
        for (int i = 0; i < WV; ++i) {
            const int u = tid + i * THREADS;
            wv_src[i] = wv_dst[i] = -1;
            if (u < g.w_units) {
                const int k = u / per_k, j = 4 * (u - k * per_k);
                if (k0 + k < k_end) {
                    wv_src[i] = k * g.cg * taps + j;
                    wv_dst[i] = k * g.wpitch + j;
                }
            }
        }
    }
    const size_t x_base = ((size_t)n0 * a.C + c_first) * HW;
    const size_t w_base = (size_t)k0 * g.cg * taps;

    float xr[NXE], wr[NWE];
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef float f32x2v __attribute__((ext_vector_type(2)));
    f32x4 xr4[NXV], wr4[NWV];
    auto load_chunk = [&](int st) {
        const int c0 = st * CC;
        if constexpr (!VEC) {
#pragma unroll
            for (int i = 0; i < XE; ++i) {
                float v = 0.0f;
                if (x_src[i] >= 0 && c0 + (int)((x_ch >> (4 * i)) & 15ull) < g.cg) v = xg[x_base + (size_t)c0 * HW + x_src[i]];
                xr[i] = v;
            }
#pragma unroll
            for (int i = 0; i < WE; ++i) {
                float v = 0.0f;
                if (w_src[i] >= 0 && c0 + (int)((w_ch[i >> 4] >> (4 * (i & 15))) & 15ull) < g.cg) v = wg[w_base + (size_t)c0 * taps + w_src[i]];
                wr[i] = v;
            }
        } else {
            const float* xc = xg + x_base + (size_t)c0 * HW;
            const float* wc = wg + w_base + (size_t)c0 * taps;
#pragma unroll
            for (int i = 0; i < XV; ++i) {
                f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                if (xv_src[i] >= 0) v = *(const f32x4*)(xc + xv_src[i]);
                xr4[i] = v;
            }
#pragma unroll
            for (int i = 0; i < WV; ++i) {
                f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                if (wv_src[i] >= 0) v = *(const f32x4*)(wc + wv_src[i]);
                wr4[i] = v;
            }
        }
    };
    auto store_chunk = [&](int buf) {
        float* xs = lds + buf * buf_floats;
        float* ws = xs + g.xfloats;
        if constexpr (!VEC) {
#pragma unroll
            for (int i = 0; i < XE; ++i)
                if (x_dst[i] >= 0) xs[x_dst[i]] = xr[i];
#pragma unroll
            for (int i = 0; i < WE; ++i)
                if (w_dst[i] >= 0) ws[w_dst[i]] = wr[i];
        } else {
#pragma unroll
            for (int i = 0; i < XV; ++i)
                if (xv_dst[i] >= 0) *(f32x4*)(xs + xv_dst[i]) = xr4[i];
#pragma unroll
            for (int i = 0; i < WV; ++i)
                if (wv_dst[i] >= 0) {                              // filter rows are 8-byte, not 16-byte aligned in LDS
                    *(f32x2v*)(ws + wv_dst[i]) = f32x2v{wr4[i][0], wr4[i][1]};
                    *(f32x2v*)(ws + wv_dst[i] + 2) = f32x2v{wr4[i][2], wr4[i][3]};
                }
        }
    };

    // ---- fragment addresses: pixel operand per tile (float offset of the tile's pixel at tap (0,0),
    //      channel `half`), filter operand per tile
    int xo[TM], wo[TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int f = (tm * WM + wm) * 32 + l32;
        int img = 0, rem = f;
        if (g.NB > 1) {
            img = f / ppi;
            rem = f - img * ppi;
        }
        const int py = rem / a.Wo, px = rem - py * a.Wo;
        xo[tm] = g.xorg + (f < npix ? ((img * g.PH + py * a.stride_h) * g.WP + px * a.stride_w) + half * g.plane : half * g.plane);
    }
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) wo[tn] = g.xfloats + ((wn * TN + tn) * 32 + l32) * g.wpitch + half * taps;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0.0f;

    // ---- zero both buffers once (pad columns are never written afterwards), then the pipeline
    for (int i = tid; i < 2 * buf_floats; i += THREADS) lds[i] = 0.0f;
    load_chunk(0);
    __syncthreads();
    store_chunk(0);
    __syncthreads();
    for (int st = 0; st < g.n_stages; ++st) {
        if (st + 1 < g.n_stages) load_chunk(st + 1);
        const float* xs = lds + (st & 1) * buf_floats;
        if constexpr (TAPS > 0) {
            constexpr int NS = (CC / 2) * TAPS;
            float fa[2][TM], fb[2][TN];
            auto read_step = [&](int set, int step) {
                const int cp = step / TAPS, tap = step % TAPS;
                constexpr int SW = TAPS == 9 ? 3 : 1;                      // filter width of the compiled sizes
                const int r = tap / SW, sx = tap - r * SW;
                const int xoff = 2 * cp * g.plane + r * a.dil_h * g.WP + sx * a.dil_w;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) fb[set][tn] = xs[wo[tn] + 2 * cp * TAPS + tap];
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) fa[set][tm] = xs[xo[tm] + xoff];
            };
            read_step(0, 0);
#pragma unroll
            for (int t = 0; t < NS; ++t) {
                if (t + 1 < NS) read_step((t + 1) & 1, t + 1);
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[t & 1][tm], fb[t & 1][tn], acc[tm][tn], 0, 0, 0);
            }
        } else {
            for (int cp = 0; cp < CC / 2; ++cp) {
                int tap = 0;
                for (int r = 0; r < a.R; ++r) {
                    for (int s = 0; s < a.S; ++s, ++tap) {
                        const int xoff = 2 * cp * g.plane + r * a.dil_h * g.WP + s * a.dil_w;
                        const int woff = 2 * cp * taps + tap;
                        float fa[TM], fb[TN];
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm) fa[tm] = xs[xo[tm] + xoff];
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn) fb[tn] = xs[wo[tn] + woff];
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                            for (int tn = 0; tn < TN; ++tn)
                                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[tm], fb[tn], acc[tm][tn], 0, 0, 0);
                    }
                }
            }
        }
        if (st + 1 < g.n_stages) store_chunk((st + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue in registers, one store.  A lane holds, per (tm, tn), filter l32 at the 16 pixels
    //      8 * q4 + 4 * half + j of the tile: four consecutive pixels per q4.
    const bool has_bn = a.bn_scale != nullptr;
    float* __restrict__ yg = (float*)a.y;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int k = k0 + (wn * TN + tn) * 32 + l32;
        if (k >= k_end) continue;
        const ChannelAffine ca = channel_affine<DT_F32>(a, k);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int f0 = (tm * WM + wm) * 32 + 8 * q4 + 4 * half;
                if (f0 >= npix) continue;
                int img = 0, rem = f0;
                if (g.NB > 1) {
                    img = f0 / ppi;
                    rem = f0 - img * ppi;
                }
                float v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = finish(acc[tm][tn][4 * q4 + j], ca, has_bn, a.act, a.alpha);
                const size_t o = ((size_t)(n0 + img) * a.K + k) * HoWo + (size_t)p0 * a.Wo + rem;
                if (f0 + 4 <= npix && rem + 4 <= ppi && ((o & 3) == 0) && (((uintptr_t)yg & 15) == 0)) {
                    *(float4*)(yg + o) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int f = f0 + j;
                        if (f < npix) {
                            int im = 0, rm = f;
                            if (g.NB > 1) {
                                im = f / ppi;
                                rm = f - im * ppi;
                            }
                            yg[((size_t)(n0 + im) * a.K + k) * HoWo + (size_t)p0 * a.Wo + rm] = v[j];
                        }
                    }
                }
            }
        }
    }
}

struct Variant {
    const char* name;
    int WM, WN, TM, TN, CC, TAPS;
    void (*kern)(ConvArgs, Geom);
    void (*kern_vec)(ConvArgs, Geom);      // vector staging, or null
};

// name: tiled_f32_<pixels per block>x<filters per block>_c<channels per chunk>[_<filter size>]
const Variant kVariants[] = {
    {"tiled_f32_256x64_c8_3x3", 4, 1, 2, 2, 8, 9, tiled_f32_kernel<4, 1, 2, 2, 8, 9, false>, tiled_f32_kernel<4, 1, 2, 2, 8, 9, true>},
    {"tiled_f32_128x64_c8_3x3", 4, 1, 1, 2, 8, 9, tiled_f32_kernel<4, 1, 1, 2, 8, 9, false>, tiled_f32_kernel<4, 1, 1, 2, 8, 9, true>},
    {"tiled_f32_256x64_c16_1x1", 4, 1, 2, 2, 16, 1, tiled_f32_kernel<4, 1, 2, 2, 16, 1, false>, tiled_f32_kernel<4, 1, 2, 2, 16, 1, true>},
    {"tiled_f32_256x64_c8", 4, 1, 2, 2, 8, 0, tiled_f32_kernel<4, 1, 2, 2, 8, 0, false>, tiled_f32_kernel<4, 1, 2, 2, 8, 0, true>},
    {"tiled_f32_128x64_c8", 4, 1, 1, 2, 8, 0, tiled_f32_kernel<4, 1, 1, 2, 8, 0, false>, tiled_f32_kernel<4, 1, 1, 2, 8, 0, true>},
    {"tiled_f32_128x32_c8", 4, 1, 1, 1, 8, 0, tiled_f32_kernel<4, 1, 1, 1, 8, 0, false>, tiled_f32_kernel<4, 1, 1, 1, 8, 0, true>},
    {"tiled_f32_128x32_c2", 4, 1, 1, 1, 2, 0, tiled_f32_kernel<4, 1, 1, 1, 2, 0, false>, nullptr},
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);
constexpr int LDS_LIMIT = 64 * 1024;        // two blocks per compute unit and room to spare

bool plan(const ConvArgs& a, const Variant& v, int NB, int TH, bool aligned16, Geom* out)
{
    const int taps = a.R * a.S;
    const int KT = v.WN * v.TN * 32, PT = v.WM * v.TM * 32;
    if (v.TAPS > 0 && (v.TAPS != taps || (v.TAPS == 9 && a.R != 3))) return false;
    if (NB < 1 || TH < 1 || NB > a.N || TH > a.Ho) return false;
    if (NB > 1 && TH != a.Ho) return false;
    if ((long long)NB * TH * a.Wo > PT) return false;
    Geom g;
    memset(&g, 0, sizeof g);
    g.NB = NB;
    g.TH = TH;
    g.PH = (TH - 1) * a.stride_h + (a.R - 1) * a.dil_h + 1;
    // every tap of every pixel must stay inside its row: the last pixel's last tap reads column
    // (Wo-1)*stride_w + (S-1)*dil_w of the padded row
    const int need = (a.Wo - 1) * a.stride_w + (a.S - 1) * a.dil_w + 1;
    g.WP = a.W + 2 * a.pad_w > need ? a.W + 2 * a.pad_w : need;
    g.cg = a.C / a.groups;
    // vector staging: 16-byte pieces of image rows and of a filter's chunk row must start on 16-byte
    // boundaries in device memory and (image rows) in LDS, and chunks must be whole
    g.vec = v.kern_vec != nullptr && aligned16 && a.W % 4 == 0 && g.cg % v.CC == 0 && (v.CC * taps) % 4 == 0 &&
            (long long)v.CC * NB * g.PH * (a.W / 4) <= (long long)XV * THREADS && (long long)KT * v.CC * taps / 4 <= (long long)WV * THREADS;
    if (g.vec) {
        g.xorg = (4 - a.pad_w % 4) % 4;                // image column 0 at float xorg + pad_w of a row: a multiple of 4
        g.WP = (g.xorg + g.WP + 3) & ~3;
        g.x_units = v.CC * NB * g.PH * (a.W / 4);
        g.w_units = KT * v.CC * taps / 4;
    }
    // a fragment read takes channel c from lanes 0-31 and channel c+1 from lanes 32-63: 32 floats from the
    // middle of one plane and 32 from the next, which share no LDS bank if planes are 32 (mod 64) floats apart
    long long plane = (long long)NB * g.PH * g.WP;
    plane += (32 - plane % 64 + 64) % 64;
    g.kg = a.K / a.groups;
    g.kb_per_group = (g.kg + KT - 1) / KT;
    g.k_blocks = g.kb_per_group * a.groups;
    g.row_blocks = (a.Ho + TH - 1) / TH;
    g.img_blocks = (a.N + NB - 1) / NB;
    g.n_stages = (g.cg + v.CC - 1) / v.CC;
    const long long x_elems = (long long)v.CC * NB * g.PH * a.W, w_elems = (long long)KT * v.CC * taps;
    if (x_elems > (long long)XE * THREADS || w_elems > (long long)WE * THREADS) return false;
    // filter fragments: lane l of each half reads row l at the same column, the halves `taps` columns
    // apart.  A pitch of 2 (mod 4) puts the 32 rows on the 32 even banks; an odd `taps` then puts the
    // other half on the odd ones.
    g.wpitch = v.CC * taps;
    while (g.wpitch % 4 != 2) ++g.wpitch;
    const long long xfloats = (long long)v.CC * plane, wfloats = (long long)KT * g.wpitch;
    if (2 * (xfloats + wfloats) * 4 > LDS_LIMIT) return false;
    if ((long long)g.row_blocks * g.img_blocks * g.k_blocks > 0x7fffffffLL) return false;
    g.plane = (int)plane;
    g.x_elems = (int)x_elems;
    g.w_elems = (int)w_elems;
    g.xfloats = (int)xfloats;
    g.wfloats = (int)wfloats;
    *out = g;
    return true;
}

}  // namespace tf32

bool tiled_f32_plan(const ConvArgs& a, const PlanEnv& env, LaunchPlan* out)
{
    static_assert(sizeof(tf32::Geom) <= sizeof(out->geom), "geometry does not fit the plan");
    if (a.dtype != DT_F32) return false;
    if (a.groups < 1 || a.C % a.groups || a.K % a.groups) return false;
    const long long xe = (long long)a.N * a.C * a.H * a.W, ye = (long long)a.N * a.K * a.Ho * a.Wo, we = (long long)a.K * (a.C / a.groups) * a.R * a.S;
    if (xe >= (1LL << 30) || ye >= (1LL << 30) || we >= (1LL << 30)) return false;   // offsets stay in int
    // tiny problems are launch latency whatever runs them; the direct kernel splits their channels over lanes
    if (!env.pin && ye * (a.C / a.groups) * a.R * a.S < (1LL << 22)) return false;
    const int HoWo = a.Ho * a.Wo;
    double best = 1e300;
    const tf32::Variant* bv = nullptr;
    tf32::Geom bg;
    for (int i = 0; i < tf32::kNumVariants; ++i) {
        const tf32::Variant& v = tf32::kVariants[i];
        if (env.pin && strcmp(env.pin, v.name) != 0) continue;
        const int PT = v.WM * v.TM * 32, KT = v.WN * v.TN * 32;
        if (a.Wo > PT) continue;
        const bool multi = HoWo <= PT;
        const int hi = multi ? PT / HoWo : PT / a.Wo;
        for (int t = hi, tried = 0; t >= 1 && tried < 8; --t) {
            tf32::Geom g;
            if (!tf32::plan(a, v, multi ? t : 1, multi ? a.Ho : t, env.aligned16, &g)) continue;
            ++tried;
            // Estimated cycles: blocks run two to a compute unit and share its matrix pipe; a block's chunk
            // costs its MFMAs (64 cycles each per wave) over a measured efficiency (on the 56x56 3x3 layer the
            // 128x64 tile runs at 1.0, 256x64 at 0.8, the loop without a compiled filter size 13 % slower)
            // plus a fixed hand-over per chunk.
            const long long blocks = (long long)g.row_blocks * g.img_blocks * g.k_blocks;
            const long long rounds = (blocks + 2LL * env.cus - 1) / (2LL * env.cus);
            // (with vector staging the 256x64 tile no longer runs short of registers: 90 against 95 us)
            const double eff = (v.TM * v.TN == 4 ? (g.vec ? 1.0 : 0.8) : v.TM * v.TN == 2 ? 1.0 : 0.7) * (v.TAPS > 0 ? 1.0 : 0.87);
            const double chunk = (v.CC / 2) * (double)(a.R * a.S) * v.TM * v.TN * 64.0 / eff + 600.0;
            const double c = (double)rounds * 2.0 * g.n_stages * chunk;
            if (c < best) {
                best = c;
                bv = &v;
                bg = g;
            }
        }
    }
    if (!bv) return false;
    out->id = KID_TILED_F32;
    out->name = bv->name;
    out->variant = (int)(bv - tf32::kVariants);
    out->grid_x = (unsigned)(bg.row_blocks * bg.img_blocks * bg.k_blocks);
    out->grid_y = 1;
    out->block = tf32::THREADS;
    out->lds = 2 * (bg.xfloats + bg.wfloats) * 4;
    memcpy(out->geom, &bg, sizeof bg);
    return true;
}

hipError_t tiled_f32_prepare()
{
    static const hipError_t status = [] {
        for (int i = 0; i < tf32::kNumVariants; ++i) {
            for (auto kern : {tf32::kVariants[i].kern, tf32::kVariants[i].kern_vec}) {
                if (!kern) continue;
                hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, tf32::LDS_LIMIT);
                if (e != hipSuccess) return e;
            }
        }
        return hipSuccess;
    }();
    return status;
}

hipError_t tiled_f32_launch(const ConvArgs& a, const LaunchPlan& p, hipStream_t s)
{
    hipError_t e = tiled_f32_prepare();
    if (e != hipSuccess) return e;
    tf32::Geom g;
    memcpy(&g, p.geom, sizeof g);
    hipLaunchKernelGGL(g.vec ? tf32::kVariants[p.variant].kern_vec : tf32::kVariants[p.variant].kern, dim3(p.grid_x), dim3(p.block), p.lds, s, a, g);
    return hipGetLastError();
}

}  // namespace cvx
