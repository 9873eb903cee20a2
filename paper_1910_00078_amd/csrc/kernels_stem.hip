// Low-channel forward convolution on bf16 / fp16 MFMA for gfx950: the "stem" layer of a CNN
// (3 input channels, 7x7 filter, stride 2) and shapes like it, where there are too few channels to
// fill an MFMA's reduction axis and the output store dominates the bytes moved.
//
// Fig. 2 of the MIOpen paper stages slices of W and I in LDS, multiplies from registers and writes O
// once; this kernel keeps that skeleton and the fused bias + activation epilogue of its Sec. V, but
// lays the reduction out along the filter WIDTH instead of the channels:
//
//   reduction index  (c, r, s') with s' = 0..7: one octet = the 8 consecutive input columns that
//                    filter row r of channel c touches (S <= 8 taps, the rest zero weights).  In NCHW
//                    those 8 columns are contiguous, so the input goes into LDS as it is -- rows of
//                    columns per (channel, input row), no transposition -- and an MFMA pixel operand
//                    is 16 contiguous bytes starting at column q*stride_w - pad_w.
//   MFMA             v_mfma_f32_32x32x16: lanes 0-31 take octet (c,r) = pair 2j, lanes 32-63 pair 2j+1.
//   alignment        the LDS row is shifted so that column -pad_w sits at element 0; with an even
//                    stride_w every operand then starts on a 4-byte boundary (two ds_read2_b32).
//                    The loader reads device memory 16 bytes at a time from column 8u - pad_w, which
//                    makes its LDS stores 16-byte aligned (device loads may be 2-byte aligned).
//   filters in LDS   [pair (c,r)][filter][8 x 16 bit], zero-filled, written once per block.
//   epilogue         bias / batch-norm / activation in registers, the tile through LDS as
//                    [filter][pixel], one 16-byte-per-lane store along the pixel axis.
#include "cvx_device.h"

#include <cstdlib>
#include <cstring>

namespace cvx {


struct StemGeom {
    int TH;            // output rows per block (tiles span the full output width)
    int PH;            // input rows a block needs: (TH-1)*stride_h + R
    int WROW;          // LDS row pitch in elements (multiple of 8, >= W + pad_w + 8)
    int UPR;           // 16-byte loader units per LDS row
    int n_units;       // C * PH * UPR
    int n_pairs;       // C * R  ((channel, filter row) pairs = octets of the reduction)
    int n_ksteps;      // ceil(n_pairs / 2)
    int row_blocks, k_blocks;
    int xbytes, wbytes;
    uint32_t wo_magic; // ceil(2^32 / Wo) for dividing pixel indices (< 65536) by Wo
    uint32_t upr_magic;
    uint32_t ph_magic;
};

__device__ __forceinline__ int div_small(int n, int d, uint32_t magic) { return d == 1 ? n : (int)__umulhi((uint32_t)n, magic); }

// ---- pieces both arrangements below share -------------------------------------------------------

// The input patch of a tile as 16-byte loader units, XU per thread of the NT threads that load: unit
// u of LDS row rowi = c*PH + patch row covers columns 8u - pad_w .. 8u - pad_w + 7.
template <int XU, int NT>
struct StemPatchLoader {
    int dst[XU], c[XU], pr[XU], col[XU];      // LDS byte offset (-1: no unit), channel, patch row, first column

    __device__ __forceinline__ void init(const ConvArgs& a, const StemGeom& g, int t)
    {
#pragma unroll
        for (int j = 0; j < XU; ++j) {
            const int ui = j * NT + t;
            dst[j] = -1;
            c[j] = pr[j] = col[j] = 0;
            if (ui < g.n_units) {
                const int rowi = div_small(ui, g.UPR, g.upr_magic);
                const int u = ui - rowi * g.UPR;
                c[j] = div_small(rowi, g.PH, g.ph_magic);
                pr[j] = rowi - c[j] * g.PH;
                col[j] = 8 * u - a.pad_w;
                dst[j] = (rowi * g.WROW + 8 * u) * 2;
            }
        }
    }
    // Issues the loads of the patch of row block rb of image n (nothing here uses a loaded value).
    __device__ __forceinline__ void load(const ConvArgs& a, const StemGeom& g, int n, int rb, u32x4 (&xv)[XU]) const
    {
        const uint16_t* __restrict__ xg = (const uint16_t*)a.x;
        const long long x_total = (long long)a.N * a.C * a.H * a.W;
        const int h_lo = rb * g.TH * a.stride_h - a.pad_h;
#pragma unroll
        for (int j = 0; j < XU; ++j) {
            xv[j] = u32x4{0u, 0u, 0u, 0u};
            const int h = h_lo + pr[j];
            if (dst[j] >= 0 && h >= 0 && h < a.H && col[j] < a.W && col[j] + 8 > 0) {
                const long long off = ((long long)(n * a.C + c[j]) * a.H + h) * a.W + col[j];
                if (off >= 0 && off + 8 <= x_total) {
                    xv[j] = *(const u32x4_a2*)(xg + off);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const long long o = off + e;
                        if (o >= 0 && o < x_total) xv[j][e >> 1] |= ((uint32_t)xg[o]) << ((e & 1) * 16);
                    }
                }
            }
        }
    }
    // Clears the columns outside [0, W) (they belong to a neighbouring row, or to nothing) and writes
    // the patch into the LDS patch buffer xs.
    __device__ __forceinline__ void store(const ConvArgs& a, unsigned char* xs, const u32x4 (&xv)[XU]) const
    {
#pragma unroll
        for (int j = 0; j < XU; ++j) {
            if (dst[j] >= 0) {
                u32x4 v = xv[j];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int cl = col[j] + e;
                    if (cl < 0 || cl >= a.W) v[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
                }
                *(u32x4*)(xs + dst[j]) = v;
            }
        }
    }
};

// Filters k0 .. k0+KT-1 into LDS at ws, by NT threads (t = 0..NT-1), WU units per thread and batch: one
// 16-byte unit per (pair = c*R + r, filter).  The S <= 8 taps of a filter row are contiguous in
// w[k][c][r][s]; one (2-byte aligned) 16-byte load fetches them, the elements past S are cleared, and the
// unit lands at [pair][filter].  Pairs past C*R (the odd one out) and filters past K are zero.  All loads
// of a batch are issued before any is used.
template <int KT, int WU, int NT>
__device__ __forceinline__ void stem_load_filters(const ConvArgs& a, const StemGeom& g, unsigned char* ws, int k0, int t)
{
    const uint16_t* __restrict__ wg = (const uint16_t*)a.w;
    const int per_k = a.C * a.R * a.S;
    const long long w_total = (long long)a.K * per_k;
    const int n_wunits = 2 * g.n_ksteps * KT;
    for (int base = 0; base < n_wunits; base += NT * WU) {
        u32x4 wv[WU];
#pragma unroll
        for (int j = 0; j < WU; ++j) {
            const int ui = base + j * NT + t;
            wv[j] = u32x4{0u, 0u, 0u, 0u};
            if (ui < n_wunits) {
                const int kl = ui % KT, pair = ui / KT;
                if (pair < g.n_pairs && k0 + kl < a.K) {
                    const long long off = (long long)(k0 + kl) * per_k + pair * a.S;
                    if (off + 8 <= w_total) {
                        wv[j] = *(const u32x4_a2*)(wg + off);
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (off + e < w_total) wv[j][e >> 1] |= ((uint32_t)wg[off + e]) << ((e & 1) * 16);
                    }
                }
            }
        }
#pragma unroll
        for (int j = 0; j < WU; ++j) {
            const int ui = base + j * NT + t;
            if (ui < n_wunits) {
                u32x4 v = wv[j];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (e >= a.S) v[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
                *(u32x4*)(ws + (size_t)ui * 16) = v;
            }
        }
    }
}

// Byte offset, inside a patch buffer, of the (channel, filter row) pair that half-wave `half` multiplies in
// each of the NKS k-steps (0 for the odd pair out, whose weights are zero).
template <int NKS>
__device__ __forceinline__ void stem_row_offsets(const ConvArgs& a, const StemGeom& g, int half, int (&rowoff)[NKS])
{
    int c = 0, r = half;
    while (r >= a.R) { r -= a.R; ++c; }
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
        rowoff[ks] = (2 * ks + half) < g.n_pairs ? ((c * g.PH + r) * g.WROW) * 2 : 0;
        r += 2;
        while (r >= a.R) { r -= a.R; ++c; }
    }
}

// The reduction with a compile-time number of k-steps, straight-line and in a pinned order: one k-step
// = two (channel, filter row) pairs, one per half-wave; after each MFMA of step ks one fragment of step
// ks+1 is read (pixels 0, the filters, then the other pixels: the order the next step's MFMAs want
// them), so the waits the compiler inserts are partial and the LDS latency hides behind the matrix pipe.
// xs: patch buffer; wl: this lane's position in the filter region; xbase: the lane's pixel operands.
template <int DT, int TM, int TN, int NKS, int KT>
__device__ __forceinline__ void stem_multiply(const unsigned char* xs, const unsigned char* wl, const int (&xbase)[TM],
                                              const int (&rowoff)[NKS], f32x16 (&acc)[TM][TN])
{
    u32x4 fa[2][TM], fb[2][TN];
    auto read_a = [&](int tm, int ks) __attribute__((always_inline)) {
        const uint32_t* p = (const uint32_t*)(xs + xbase[tm] + rowoff[ks]);   // 4-byte aligned
        return u32x4{p[0], p[1], p[2], p[3]};
    };
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) fb[0][tn] = *(const u32x4*)(wl + tn * 32 * 16);
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) fa[0][tm] = read_a(tm, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
        const int b = ks & 1, nb = b ^ 1;
        const bool more_k = ks + 1 < NKS;
        int issued = 0;
        auto read_next = [&]() __attribute__((always_inline)) {
            if (issued == 0) fa[nb][0] = read_a(0, ks + 1);
            else if (issued <= TN) fb[nb][issued - 1] = *(const u32x4*)(wl + ((ks + 1) * 2 * KT + (issued - 1) * 32) * 16);
            else fa[nb][issued - TN] = read_a(issued - TN, ks + 1);
            ++issued;
        };
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                acc[tm][tn] = mfma_32x32x16<DT>(fa[b][tm], fb[b][tn], acc[tm][tn]);
                __builtin_amdgcn_sched_barrier(0);
                if (more_k && issued < TM + TN) {
                    read_next();
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < TM + TN; ++j) {
            if (more_k && issued < TM + TN) {
                read_next();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
}

// Block: 4 waves, PT = 4*TM*32 pixels (TH full output rows) x KT = TN*32 filters.  Blocks are
// persistent: block b works through tiles b, b + gridDim.x, ... with the filters resident in LDS and
// the loop software-pipelined -- the input patch of the next tile is fetched into registers while the
// current one is multiplied, and the stores of the current tile drain while the next one starts.
//
// LDS map: filters [pair][KT][8] | input patch [c][patch row][WROW] | output tile [KT][PT + 8].
template <int DT, int TM, int TN, int NKS>
__global__ void __launch_bounds__(256) stem_kernel(ConvArgs a, StemGeom g)
{
    constexpr int THREADS = 256;
    constexpr int WAVES = 4;
    constexpr int PT = WAVES * TM * 32;
    constexpr int KT = TN * 32;
    constexpr int PTP = PT + 8;
    constexpr int XU = 4;                            // input loader units per thread (host guarantees enough)
    constexpr int WU = 6;                            // filter loader units per thread and batch
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    CVX_TRACE_MARK(0);
    warm_kernel_arguments<sizeof(ConvArgs) + sizeof(StemGeom)>();
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int HoWo = a.Ho * a.Wo;
    uint16_t* __restrict__ yg = (uint16_t*)a.y;

    unsigned char* ws = smem;                            // filters
    unsigned char* xs = smem + g.wbytes;                 // input patch
    uint16_t* ot = (uint16_t*)(smem + g.wbytes + g.xbytes);   // output tile

    const int tiles_per_kb = a.N * g.row_blocks;
    const int n_tiles = tiles_per_kb * g.k_blocks;

    // ---- tile-independent bookkeeping
    StemPatchLoader<XU, THREADS> patch;
    patch.init(a, g, tid);
    // operand addresses: byte offset of (patch row py*stride_h, column index px*stride_w) per pixel tile
    int xbase[TM];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int f = (tm * WAVES + wave) * 32 + l32;         // pixel tiles dealt round-robin to the waves
        const int py = div_small(f, a.Wo, g.wo_magic);
        const int px = f - py * a.Wo;
        xbase[tm] = f < g.TH * a.Wo ? ((py * a.stride_h) * g.WROW + px * a.stride_w) * 2 : 0;
    }
    const bool has_bn = a.bn_scale != nullptr;
    // With a compile-time number of k-steps (NKS > 0) the byte offset of every step's (channel, filter
    // row) pair is worked out once; the reduction loop is then straight-line code.
    int rowoff[NKS > 0 ? NKS : 1];
    if constexpr (NKS > 0) stem_row_offsets<NKS>(a, g, half, rowoff);

    auto load_patch = [&](int tile, u32x4 (&xv)[XU]) __attribute__((always_inline)) {
        const int pt = tile % tiles_per_kb;
        const int n = pt / g.row_blocks;
        patch.load(a, g, n, pt - n * g.row_blocks, xv);
    };
    int tile = blockIdx.x;
    if (tile >= n_tiles) return;
    int cur_kb = -1;
    ChannelAffine ca[TN];                            // epilogue constants of this lane's filters
    u32x4 xv[XU];

    // Brings a tile's patch (already in xv) into LDS, and the filters and epilogue constants if the
    // filter block changed (once per block unless K > KT).
    auto enter_tile = [&](int tl) __attribute__((always_inline)) {
        patch.store(a, xs, xv);
        const int kb = tl / tiles_per_kb;
        if (kb != cur_kb) {
            stem_load_filters<KT, WU, THREADS>(a, g, ws, kb * KT, tid);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) ca[tn] = channel_affine<DT>(a, min(kb * KT + tn * 32 + l32, a.K - 1));
            cur_kb = kb;
        }
    };

    load_patch(tile, xv);
    enter_tile(tile);
    int pass = 0;                                    // tiles this block has finished
    (void)pass;
    // Phase stamps are taken on the block's fourth tile: a steady-state pass, not the first or last.
#define STEM_MARK(s) do { if (pass == 3) CVX_TRACE_MARK(s); } while (0)

    for (; tile < n_tiles; tile += gridDim.x) {
        const int kb = tile / tiles_per_kb;
        const int pt = tile - kb * tiles_per_kb;
        const int n = pt / g.row_blocks;
        const int rb = pt - n * g.row_blocks;
        const int k0 = kb * KT;
        const int p0 = rb * g.TH;
        const int npix = min(g.TH, a.Ho - p0) * a.Wo;
        const bool wave_on = wave < ((npix + 31) >> 5);
        const bool more = tile + gridDim.x < n_tiles;

        // (1) patch and filters of this tile are in LDS (written before the previous pass's stores)
        __syncthreads();
        STEM_MARK(2);

        // (2) start fetching the next tile's patch.  No device load is consumed between here and
        //     (5): one would make the wave wait for this prefetch.
        if (more) load_patch(tile + gridDim.x, xv);

        // (3) multiply.  One k-step = two (channel, filter row) pairs, one per half-wave; the fragments of
        //     step ks+1 are read before the MFMAs of step ks are issued (two register sets).
        f32x16 acc[TM][TN];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const float seed = has_bn ? 0.0f : ca[tn].add;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[tm][tn][r] = seed;
            }
        if (wave_on) {
            if constexpr (NKS > 0) {
                stem_multiply<DT, TM, TN, NKS, KT>(xs, ws + (size_t)(half * KT + l32) * 16, xbase, rowoff, acc);
            } else {
            int pr = half;                               // this half-wave's pair index
            int c = 0, r = half;
            while (r >= a.R) { r -= a.R; ++c; }
            auto read_step = [&](u32x4 (&fa)[TM], u32x4 (&fb)[TN]) __attribute__((always_inline)) {
                const bool live = pr < g.n_pairs;        // the odd pair out multiplies zero weights
                const int rowoff = live ? ((c * g.PH + r) * g.WROW) * 2 : 0;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    fb[tn] = *(const u32x4*)(ws + ((size_t)pr * KT + tn * 32 + l32) * 16);   // dead pairs hold zeros
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    const uint32_t* p = (const uint32_t*)(xs + xbase[tm] + rowoff);   // 4-byte aligned
                    fa[tm] = u32x4{p[0], p[1], p[2], p[3]};
                }
                pr += 2;
                r += 2;
                while (r >= a.R) { r -= a.R; ++c; }
            };
            auto mul_step = [&](const u32x4 (&fa)[TM], const u32x4 (&fb)[TN]) __attribute__((always_inline)) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) acc[tm][tn] = mfma_32x32x16<DT>(fa[tm], fb[tn], acc[tm][tn]);
            };
            u32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
            read_step(fa0, fb0);
            for (int ks = 0; ks < g.n_ksteps; ks += 2) {
                if (ks + 1 < g.n_ksteps) read_step(fa1, fb1);
                __builtin_amdgcn_sched_barrier(0);
                mul_step(fa0, fb0);
                __builtin_amdgcn_sched_barrier(0);
                if (ks + 1 < g.n_ksteps) {
                    if (ks + 2 < g.n_ksteps) read_step(fa0, fb0);
                    __builtin_amdgcn_sched_barrier(0);
                    mul_step(fa1, fb1);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            }
        }
        STEM_MARK(5);

        // (4) epilogue part 1: registers -> LDS as [filter][pixel] in the output type.  The output tile
        //     has its own LDS region; the previous pass's store loop finished reading it before (1).
        if (wave_on) {
            auto stage_out = [&](auto&& act_fn) __attribute__((always_inline)) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const int kl = tn * 32 + l32;
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            float v[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const float t = acc[tm][tn][4 * q4 + j];
                                v[j] = act_fn(has_bn ? fmaf(t, ca[tn].mul, ca[tn].add) : t);
                            }
                            const int f = (tm * WAVES + wave) * 32 + 8 * q4 + 4 * half;
                            *(uint2*)(ot + kl * PTP + f) = make_uint2(pack2<DT>(v[0], v[1]), pack2<DT>(v[2], v[3]));
                        }
                    }
                }
            };
            if (a.act == ACT_RELU) stage_out([](float t) { return fmaxf(t, 0.0f); });
            else if (a.act == ACT_IDENTITY) stage_out([](float t) { return t; });
            else stage_out([&](float t) { return activate(t, a.act, a.alpha); });
        }
        __syncthreads();                             // output tile complete; all reads of xs / ws done
        STEM_MARK(6);

        // (5) the next tile's patch goes into LDS now, BEFORE this tile's stores are issued: loads and
        //     stores share one in-order counter, so waiting for the patch after the stores would wait
        //     for the stores to drain as well.
        if (more) enter_tile(tile + gridDim.x);
        STEM_MARK(7);

        // (6) epilogue part 2: the single store, 16 bytes per lane along the pixel axis
        {
            constexpr int CH = PT / 8;
            constexpr int RSTEP = THREADS / CH;
            constexpr int NPASS = (KT + RSTEP - 1) / RSTEP;
            const int chunk = tid % CH, row0 = tid / CH;
            const int f0 = chunk * 8;
            if (f0 < npix) {
                const bool whole = f0 + 8 <= npix;
                const size_t obase = ((size_t)n * a.K + k0) * HoWo + (size_t)p0 * a.Wo + f0;
                constexpr int GRP = NPASS >= 4 ? 4 : NPASS;
                for (int p = 0; p < NPASS; p += GRP) {
                    u32x4 v[GRP];
#pragma unroll
                    for (int j = 0; j < GRP; ++j) v[j] = *(const u32x4*)(ot + min(row0 + (p + j) * RSTEP, KT - 1) * PTP + f0);
#pragma unroll
                    for (int j = 0; j < GRP; ++j) {
                        const int kl = row0 + (p + j) * RSTEP;
                        if (kl < KT && k0 + kl < a.K) {
                            uint16_t* dst = yg + obase + (size_t)kl * HoWo;
                            if (whole) {
                                // streaming store: lines left dirty in L2 would have to be written back at the end of the kernel
                                __builtin_nontemporal_store(v[j], (u32x4_a2*)dst);
                            } else {
#pragma unroll
                                for (int e = 0; e < 8; ++e)
                                    if (f0 + e < npix) dst[e] = (uint16_t)(v[j][e >> 1] >> ((e & 1) * 16));
                            }
                        }
                    }
                }
            }
        }
        STEM_MARK(15);
        ++pass;
    }
#undef STEM_MARK
}

// ------------------------------------------------------------------------------------------------
// Streaming arrangement of the same computation, for layers whose filters fit one block (K <= 64):
// the roles are split so that nothing but one hand-over per tile is block-wide.
//
//   loader waves (4)    fetch the input patch of tile i+2 into registers, and write the patch of tile
//                       i+1 (fetched a tile earlier) into the other of two LDS patch buffers, while
//                       the multiply waves work on tile i;
//   multiply waves (8)  64 pixels x 64 filters each: fragments from the current patch buffer and the
//                       resident filters, MFMA, epilogue in registers, then each wave stages its own
//                       results through a private LDS patch and stores 128-byte rows itself.  They
//                       never wait for a device load, and the loaders never wait for a store.
//
// LDS map: filters | patch buffer 0 | patch buffer 1 | one output patch [32 filters][64 px + 4] per wave.
constexpr int STREAM_NCW = 8, STREAM_NLW = 4;   // 12 waves = 3 per SIMD, one block per CU
constexpr int STREAM_THREADS = (STREAM_NCW + STREAM_NLW) * 64;
constexpr int STREAM_XU = 5;                  // input loader units per loader thread
constexpr int STREAM_OPITCH = 136;            // bytes per filter row of an output patch: 64 pixels + 4 (bank spread)
constexpr int STREAM_PATCH = 32 * STREAM_OPITCH;

template <int DT, int NKS>
__global__ void __launch_bounds__(STREAM_THREADS) stem_stream_kernel(ConvArgs a, StemGeom g)
{
    constexpr int TM = 2, TN = 2;
    constexpr int NCW = STREAM_NCW, THREADS = STREAM_THREADS, LTHREADS = STREAM_NLW * 64;
    constexpr int PT = NCW * TM * 32;
    constexpr int KT = TN * 32;
    constexpr int XU = STREAM_XU;
    constexpr int WU = 4;
    constexpr int OPITCH = STREAM_OPITCH;
    static_assert(NKS > 0, "the streaming arrangement is built for a compile-time reduction length");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    CVX_TRACE_MARK(0);
    warm_kernel_arguments<sizeof(ConvArgs) + sizeof(StemGeom)>();
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int HoWo = a.Ho * a.Wo;

    unsigned char* ws = smem;                                        // filters [pair][KT] x 16 bytes
    unsigned char* xs0 = smem + g.wbytes;                            // two patch buffers
    const int n_tiles = a.N * g.row_blocks;                          // one filter block: K <= KT
    if ((int)blockIdx.x >= n_tiles) return;
    const int n_my = (n_tiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;   // tiles of this block

    auto bar = []() __attribute__((always_inline)) { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

    if (wave >= NCW) {
        // =========================================================================================
        // loader waves
        // =========================================================================================
        const int lt = tid - NCW * 64;
        StemPatchLoader<XU, LTHREADS> patch;
        patch.init(a, g, lt);
        u32x4 xv[XU];
        auto load_patch = [&](int i) __attribute__((always_inline)) {
            const int tile = (int)blockIdx.x + i * (int)gridDim.x;
            const int n = tile / g.row_blocks;
            patch.load(a, g, n, tile - n * g.row_blocks, xv);
        };
        auto store_patch = [&](int buf) __attribute__((always_inline)) { patch.store(a, xs0 + buf * g.xbytes, xv); };
        load_patch(0);
        store_patch(0);
        bar();                                                       // filters and the first patch are in LDS
        if (n_my > 1) load_patch(1);
        for (int i = 0; i < n_my; ++i) {
            if (i + 1 < n_my) {
                store_patch((i + 1) & 1);                            // that buffer was multiplied a pass ago
                if (i + 2 < n_my) load_patch(i + 2);
            }
            bar();
        }
    } else {
        // =========================================================================================
        // multiply waves
        // =========================================================================================
        const int l32 = lane & 31, half = lane >> 5;
        const bool has_bn = a.bn_scale != nullptr;
        uint16_t* __restrict__ yg = (uint16_t*)a.y;
        // operand addresses: the wave owns pixels [wave*64, wave*64 + 64) of the tile
        int xbase[TM];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int f = (wave * TM + tm) * 32 + l32;
            const int py = div_small(f, a.Wo, g.wo_magic);
            const int px = f - py * a.Wo;
            xbase[tm] = f < g.TH * a.Wo ? ((py * a.stride_h) * g.WROW + px * a.stride_w) * 2 : 0;
        }
        int rowoff[NKS];
        stem_row_offsets<NKS>(a, g, half, rowoff);
        // filters, once per block, by the multiply waves (the loaders are already fetching the first patch)
        stem_load_filters<KT, WU, NCW * 64>(a, g, ws, 0, tid);
        ChannelAffine ca[TN];
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) ca[tn] = channel_affine<DT>(a, min(tn * 32 + l32, a.K - 1));
        unsigned char* ow = smem + g.wbytes + 2 * g.xbytes + wave * STREAM_PATCH;
        const unsigned char* wl = ws + (size_t)(half * KT + l32) * 16;
        // identity, ReLU and leaky ReLU are one formula, max(v,0) + slope*min(v,0); tanh and logistic are
        // applied to the accumulators in a separate pass, after which the formula runs as the identity
        const bool slow_act = a.act == ACT_TANH || a.act == ACT_LOGISTIC;
        const float neg_slope = (a.act == ACT_IDENTITY || slow_act) ? 1.0f : (a.act == ACT_LEAKY_RELU ? a.alpha : 0.0f);
        const bool bn_inline = has_bn && !slow_act;
        const bool packed_act = !has_bn && (a.act == ACT_RELU || a.act == ACT_IDENTITY);
        const uint32_t floor2 = packed_floor(a.act == ACT_RELU);

        bar();                                                       // filters and the first patch are in LDS
        for (int i = 0; i < n_my; ++i) {
            const int tile = (int)blockIdx.x + i * (int)gridDim.x;
            const int n = tile / g.row_blocks;
            const int rb = tile - n * g.row_blocks;
            const int p0 = rb * g.TH;
            const int npix = min(g.TH, a.Ho - p0) * a.Wo;
            const unsigned char* xs = xs0 + (i & 1) * g.xbytes;
            const bool wave_on = wave * TM * 32 < npix;

            f32x16 acc[TM][TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const float seed = has_bn ? 0.0f : ca[tn].add;
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[tm][tn][r] = seed;
                }
            if (wave_on) {
                stem_multiply<DT, TM, TN, NKS, KT>(xs, wl, xbase, rowoff, acc);

                // epilogue: 32 filters at a time through the wave's own patch, then 16 bytes per lane
                // along the pixel axis (the tile is TH whole output rows: its pixels are contiguous in y)
                if (slow_act) {
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const float t = acc[tm][tn][r];
                                acc[tm][tn][r] = activate(has_bn ? fmaf(t, ca[tn].mul, ca[tn].add) : t, a.act, a.alpha);
                            }
                }
                const int P0 = wave * (TM * 32) + (lane & 7) * 8;     // this lane's 8 pixels of the tile
                const bool any = P0 < npix, whole = P0 + 8 <= npix;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    if (packed_act) {
                        // bias + ReLU / identity: round, then ReLU on the packed pair, 1 instruction per value
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                            for (int q4 = 0; q4 < 4; ++q4) {
                                const f32x16& t = acc[tm][tn];
                                *(uint2*)(ow + l32 * OPITCH + (tm * 32 + 8 * q4 + 4 * half) * 2) =
                                    make_uint2(max_packed(pack2<DT>(t[4 * q4], t[4 * q4 + 1]), floor2),
                                               max_packed(pack2<DT>(t[4 * q4 + 2], t[4 * q4 + 3]), floor2));
                            }
                    } else {
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                            for (int q4 = 0; q4 < 4; ++q4) {
                                float v[4];
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    float t = acc[tm][tn][4 * q4 + j];
                                    if (bn_inline) t = fmaf(t, ca[tn].mul, ca[tn].add);
                                    v[j] = fmaf(neg_slope, fminf(t, 0.0f), fmaxf(t, 0.0f));
                                }
                                *(uint2*)(ow + l32 * OPITCH + (tm * 32 + 8 * q4 + 4 * half) * 2) =
                                    make_uint2(pack2<DT>(v[0], v[1]), pack2<DT>(v[2], v[3]));
                            }
                    }
                    u32x4 o[4];
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const unsigned char* p = ow + (r4 * 8 + (lane >> 3)) * OPITCH + (lane & 7) * 16;
                        const uint2 lo = *(const uint2*)p, hi = *(const uint2*)(p + 8);
                        o[r4] = u32x4{lo.x, lo.y, hi.x, hi.y};
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    const size_t obase = ((size_t)n * a.K + tn * 32) * HoWo + (size_t)p0 * a.Wo + P0;
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const int kl = r4 * 8 + (lane >> 3);
                        if (any && tn * 32 + kl < a.K) {
                            uint16_t* dst = yg + obase + (size_t)kl * HoWo;
                            if (whole) {
                                // streaming store: lines left dirty in L2 would have to be written back at the end of the kernel
                                __builtin_nontemporal_store(o[r4], (u32x4_a2*)dst);
                            } else {
#pragma unroll
                                for (int e = 0; e < 8; ++e)
                                    if (P0 + e < npix) dst[e] = (uint16_t)(o[r4][e >> 1] >> ((e & 1) * 16));
                            }
                        }
                    }
                }
            }
            if (i < 6) CVX_TRACE_MARK(2 + i);
            bar();
        }
        CVX_TRACE_MARK(15);
    }
}

// ------------------------------------------------------------------------------------------------
namespace {

constexpr int STEM_LDS_LIMIT = 80 * 1024;     // two blocks per CU
constexpr int STREAM_LDS_LIMIT = 160 * 1024;  // the streaming arrangement runs one block per CU

struct StemVariant {
    const char* name;
    int TM, TN, NKS;
    int stream;        // 1: streaming arrangement (loader waves + multiply waves), K <= 64
    void (*kern_bf16)(ConvArgs, StemGeom);
    void (*kern_f16)(ConvArgs, StemGeom);
};

const StemVariant kStem[] = {
    {"stem_stream_512x64_k11", 2, 2, 11, 1, stem_stream_kernel<DT_BF16, 11>, stem_stream_kernel<DT_F16, 11>},
    // reduction fully unrolled for 3 channels x 7 filter rows (11 k-steps)
    {"stem_256x64_k11", 2, 2, 11, 0, stem_kernel<DT_BF16, 2, 2, 11>, stem_kernel<DT_F16, 2, 2, 11>},
    {"stem_128x64_k11", 1, 2, 11, 0, stem_kernel<DT_BF16, 1, 2, 11>, stem_kernel<DT_F16, 1, 2, 11>},
    // any C*R: run-time reduction loop
    {"stem_256x64", 2, 2, 0, 0, stem_kernel<DT_BF16, 2, 2, 0>, stem_kernel<DT_F16, 2, 2, 0>},
    {"stem_128x64", 1, 2, 0, 0, stem_kernel<DT_BF16, 1, 2, 0>, stem_kernel<DT_F16, 1, 2, 0>},
};
constexpr int kNumStem = sizeof(kStem) / sizeof(kStem[0]);

int stem_lds(const StemVariant& v, const StemGeom& g)
{
    if (v.stream) return g.wbytes + 2 * g.xbytes + STREAM_NCW * STREAM_PATCH;
    const int PT = 4 * v.TM * 32, KT = v.TN * 32;
    return g.xbytes + g.wbytes + KT * (PT + 8) * 2;
}

bool stem_choose(const ConvArgs& a, const PlanEnv& env, const StemVariant** vout, StemGeom* gout)
{
    if (a.dtype != DT_BF16 && a.dtype != DT_F16) return false;
    if (a.groups != 1) return false;
    if (a.C > 4 || a.S > 8 || a.R > 16) return false;              // low-channel layers only
    if (a.dil_h != 1 || a.dil_w != 1) return false;
    if ((a.stride_w & 1) || a.stride_w > 8) return false;          // operands must start 4-byte aligned
    if (a.Wo >= 32768 || a.W >= 32768) return false;
    const long long xbytes = (long long)a.N * a.C * a.H * a.W * 2, ybytes = (long long)a.N * a.K * a.Ho * a.Wo * 2;
    if (xbytes >= (1LL << 31) || ybytes >= (1LL << 31)) return false;
    if (!env.aligned16) return false;
    const char* want = env.pin;                                     // developer pin: variant name
    for (const StemVariant& v : kStem) {
        const int PT = (v.stream ? STREAM_NCW : 4) * v.TM * 32, KT = v.TN * 32;
        if (want && *want && strcmp(want, v.name) != 0) continue;
        if (v.NKS > 0 && (a.C * a.R + 1) / 2 != v.NKS) continue;
        if (a.Wo > PT) continue;
        StemGeom g;
        g.TH = PT / a.Wo;
        if (g.TH > a.Ho) g.TH = a.Ho;
        g.PH = (g.TH - 1) * a.stride_h + a.R;
        // the last pixel's operand reads 8 columns from (Wo-1)*stride_w; rows are zero-filled up to WROW
        const int need = (a.Wo - 1) * a.stride_w + 8;
        const int have = a.W + a.pad_w;
        g.WROW = ((need > have ? need : have) + 7) & ~7;
        g.UPR = g.WROW / 8;
        g.n_units = a.C * g.PH * g.UPR;
        g.n_pairs = a.C * a.R;
        g.n_ksteps = (g.n_pairs + 1) / 2;
        g.row_blocks = (a.Ho + g.TH - 1) / g.TH;
        g.k_blocks = (a.K + KT - 1) / KT;
        g.xbytes = a.C * g.PH * g.WROW * 2;
        g.wbytes = 2 * g.n_ksteps * KT * 16;
        if (stem_lds(v, g) > (v.stream ? STREAM_LDS_LIMIT : STEM_LDS_LIMIT)) continue;
        if (v.stream) {
            if (g.k_blocks != 1 || g.n_units > STREAM_XU * STREAM_NLW * 64) continue;
        } else if (g.n_units > 4 * 256) {
            continue;                                              // 4 loader units per thread
        }
        if ((long long)a.N * g.row_blocks * g.k_blocks > 0x7fffffffLL) continue;
        g.wo_magic = a.Wo > 1 ? (uint32_t)(((1ull << 32) + a.Wo - 1) / a.Wo) : 0u;
        g.upr_magic = g.UPR > 1 ? (uint32_t)(((1ull << 32) + g.UPR - 1) / g.UPR) : 0u;
        g.ph_magic = g.PH > 1 ? (uint32_t)(((1ull << 32) + g.PH - 1) / g.PH) : 0u;
        // prefer the variant that wastes fewer pixel slots
        const int used = g.TH * a.Wo;
        if (used * 4 < PT * 3 && v.TM > 1) continue;       // mostly empty: a smaller tile follows in the table
        *vout = &v;
        *gout = g;
        return true;
    }
    return false;
}

}  // namespace

#ifdef CVX_PHASE_TRACE
extern "C" int cvx_debug_set_phase_trace_stem(unsigned long long* device_buffer)
{
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_phase_trace), &device_buffer, sizeof(device_buffer));
}
#endif

bool stem_plan(const ConvArgs& a, const PlanEnv& env, LaunchPlan* out)
{
    static_assert(sizeof(StemGeom) <= sizeof(out->geom), "geometry does not fit the plan");
    const StemVariant* v;
    StemGeom g;
    if (!stem_choose(a, env, &v, &g)) return false;
    const int lds = stem_lds(*v, g);
    // persistent blocks: as many as stay resident at once (LDS decides), each striding through the tiles
    const long long tiles = (long long)a.N * g.row_blocks * g.k_blocks;
    int per_cu = (160 * 1024) / lds;
    if (per_cu > 4) per_cu = 4;
    if (per_cu < 1) per_cu = 1;
    long long blocks = (long long)env.cus * per_cu;
    if (blocks > tiles) blocks = tiles;
    out->id = KID_STEM;
    out->name = v->name;
    out->variant = (int)(v - kStem);
    out->grid_x = (unsigned)blocks;
    out->grid_y = 1;
    out->block = v->stream ? STREAM_THREADS : 256;
    out->lds = lds;
    memcpy(out->geom, &g, sizeof g);
    return true;
}

hipError_t stem_prepare()
{
    static const hipError_t status = [] {
        for (int i = 0; i < kNumStem; ++i) {
            for (auto kern : {kStem[i].kern_bf16, kStem[i].kern_f16}) {
                hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                   kStem[i].stream ? STREAM_LDS_LIMIT : STEM_LDS_LIMIT);
                if (e != hipSuccess) return e;
            }
        }
        return hipSuccess;
    }();
    return status;
}

hipError_t stem_launch(const ConvArgs& a, const LaunchPlan& p, hipStream_t s)
{
    hipError_t e = stem_prepare();
    if (e != hipSuccess) return e;
    const StemVariant& v = kStem[p.variant];
    StemGeom g;
    memcpy(&g, p.geom, sizeof g);
    auto kern = a.dtype == DT_BF16 ? v.kern_bf16 : v.kern_f16;
    hipLaunchKernelGGL(kern, dim3(p.grid_x), dim3(p.block), p.lds, s, a, g);
    return hipGetLastError();
}

}  // namespace cvx
