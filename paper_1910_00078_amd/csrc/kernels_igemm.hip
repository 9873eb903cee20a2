// Implicit-GEMM forward convolution on bf16 / fp16 MFMA for gfx950 (MI355X).
//
// The structure is the one Fig. 2 of the MIOpen paper draws for its composable-kernel implicit
// GEMM -- blockwise slices of W and I from device memory into LDS, threadwise slices from LDS into
// registers, accumulation of O in registers over (C-chunk, Y, X), one copy of O back to device
// memory -- with the bias + activation epilogue of Sec. V applied to the accumulators before that
// single store.  The mapping onto the hardware is this library's own:
//
//   GEMM view        D[k][pix] = sum_{tap, c} Wt[k][tap][c] * X[pix @ tap][c]
//   MFMA             v_mfma_f32_32x32x16 (bf16 or f16 in, fp32 accumulate): A = 32 filters x 16
//                    channels, B = 16 channels x 32 pixels; a lane supplies 8 consecutive channels.
//   Input in LDS     channel-octet major: [octet][image][flat (h,w) element] with 16 bytes (8
//                    channels) per element, so an MFMA operand is one ds_read_b128 and the filter
//                    taps are plain address offsets.  NCHW keeps W contiguous, channels strided,
//                    so the loader reads 8 channel rows with 16-byte loads along W and transposes
//                    8x8 in registers (v_perm_b32) before 8 ds_write_b128.
//   Padding          rows outside the image are zero-filled by the loader; columns outside the
//                    image are redirected at read time to a 16-byte slot of zeros.
//   Filters in LDS   [tap][octet][filter] x 16 bytes, transposed in registers the same way.
//   Pipeline         two LDS stage buffers; the global loads of the next stage (of the next two, in
//                    the producers' common-case loop) are in flight while stage s is multiplied.
#include "cvx_device.h"

#include <cstdio>
#include <type_traits>
#include <cstdlib>
#include <cstring>

namespace cvx {

typedef __attribute__((address_space(3))) unsigned char* lds_ptr_t;

// Division of small non-negative integers by a runtime divisor chosen on the host: q = n / d for
// n, d < 65536 via one multiply-high (m = ceil(2^32 / d); exact while n * d < 2^32).
struct FastDiv {
    uint32_t m, d;
    __device__ __forceinline__ int div(int n) const { return d == 1u ? n : (int)__umulhi((uint32_t)n, m); }
};

constexpr int TRASH_BYTES = 64 * 16;

struct IgemmGeom {
    int NB;          // images per pixel tile
    int TH;          // output rows per pixel tile (tiles span the full output width)
    int PH;          // input rows a tile needs: (TH-1)*stride_h + (R-1)*dil_h + 1
    int WP;          // LDS row pitch in elements: W + 2*pad_w rounded up to a multiple of 8 (pad columns stay zero)
    int UPI;         // loader units (8 flat elements x 8 channels) per (octet, image)
    int SLOTS;       // logical LDS elements per (octet, image) = PH * WP
    int PSLOTS;      // physical ones: one spare 16-byte slot after every 8 (see lds_slot)
    int row_blocks, img_blocks, k_blocks;   // k_blocks counts the filter blocks of all groups
    int cg, kg, kb_per_group;              // channels and filters per group (Sec. IV-A grouped convolution); filter blocks per group
    int xcd_kparts;  // the 8 XCDs split the tile grid into (8 / xcd_kparts) pixel-block ranges x xcd_kparts filter-block ranges; 0: plain order
    int xcd_kshift;  // log2(xcd_kparts)
    int xcd_ppx;     // pixel blocks per XCD (filter blocks per XCD: by_kpx.d)
    int n_stages;    // ceil(C / CC)
    int a_units;     // input loader units per stage
    int b_units;     // filter loader units per stage (register-transposed path)
    int xbytes, wbytes;   // LDS bytes per stage for input and filters
    int flat;        // output staging: 0 = [filter][pixel] tile; 1, 2 = the tile's run of y, image by image (see the epilogue)
    int flat_pitch;  // elements per image of that staging
    FastDiv by_wo, by_w, by_upi, by_nb, by_kblocks, by_rowblocks, by_howo, by_kpx;
};

// 16-byte load of 8 consecutive 16-bit elements starting at element offset `off` of a tensor with
// `total` elements; elements outside the tensor read as zero.  Addresses are only 2-byte aligned.
__device__ __forceinline__ u32x4 load8(const uint16_t* base, long long off, long long total)
{
    if (off >= 0 && off + 8 <= total) return *(const u32x4_a2*)(base + off);
    u32x4 v = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const long long o = off + e;
        if (o >= 0 && o < total) v[e >> 1] |= ((uint32_t)base[o]) << ((e & 1) * 16);
    }
    return v;
}

// result = (half `hb` of b) | (half `ha` of a) << 16
__device__ __forceinline__ uint32_t pack_halves(uint32_t a, int ha, uint32_t b, int hb)
{
    const uint32_t sel = ((ha ? 0x0706u : 0x0504u) << 16) | (hb ? 0x0302u : 0x0100u);
    return __builtin_amdgcn_perm(a, b, sel);
}

// Physical position of logical element `s` of an (octet, image) region.  The loader's lanes each
// own 8 consecutive elements and write element e of all of them in one instruction, i.e. a lane
// stride of 8 slots = 128 bytes, which would put 32 lanes on the same 4 LDS banks.  One spare slot
// after every 8 makes that stride 9 slots, which walks through all bank groups; rows of 32
// consecutive elements (what an MFMA fragment read touches) stay spread as well.  Because the row
// pitch WP is a multiple of 8, moving by whole rows is still a constant byte offset (18 * WP).
__device__ __forceinline__ int lds_slot(int s) { return s + (s >> 3); }

// LDS map (bytes): two stage buffers from offset 16, each an input region (xbytes, whose last
// TRASH_BYTES are one 16-byte trash slot per lane for loader writes that must not land in the image,
// so that no two lanes of a write instruction share an address) followed by a filter region
// (wbytes).  After the last stage the same memory holds the output tile for the store.
//
// The block is split by role.  The first WM*WN waves are consumers: they own the accumulators and
// do nothing in the main loop but read fragments from LDS and issue MFMAs.  The next NPW waves are
// producers: they transpose and write stage s+1 into LDS, and fetch a later stage from device
// memory, while the consumers multiply stage s.  One consumer and one producer wave share each SIMD, so the
// producers' vector-ALU and memory work runs in the shadow of the matrix pipe.  One s_barrier per
// stage hands a finished buffer from producers to consumers and a drained one back.
// 8: four producer waves for the input and four for the filters; 4: four that do both (kernels whose
// registers do not allow three waves per SIMD: 4x2 register tiles, or several 3x3 loader units per thread).
__host__ __device__ constexpr int igemm_producer_waves(int TM, int TN, int TAPS, int UA, int UB)
{
    return (TM * TN <= 4 && !(TAPS == 9 && (UA > 1 || UB > 1))) ? 8 : 4;
}

// Filter region of a stage: [tap][octet][filter] x 16 bytes.  The loader's lanes are dealt octet-fastest, so
// the 8 lanes of one 128-byte beat of a write differ in their octet; with octets exactly KT * 16 bytes apart
// (a multiple of 128) they would all land on the same banks.  A skew of 128 / OCT bytes per octet spreads
// them; the consumers' fragment reads (32 consecutive filters of one octet) stay contiguous.
__host__ __device__ constexpr int igemm_filter_octet_pitch(int KT, int OCT)
{
    return KT * 16 + (OCT > 1 ? (128 / OCT < 16 ? 16 : 128 / OCT) : 0);
}

template <int DT, int WM, int WN, int TM, int TN, int CC, int TAPS, int UA, int UB>
__global__ void __launch_bounds__((WM * WN + igemm_producer_waves(TM, TN, TAPS, UA, UB)) * 64)
igemm_kernel(ConvArgs a, IgemmGeom g)
{
    constexpr int NCW = WM * WN;           // consumer waves
    // Producer waves.  Kernels with 2x2 register tiles leave room for twelve waves per block (three per
    // SIMD, 168 registers each): four producer waves load the input and four more the filters, which
    // halves each producer's chain of loads, transposes and LDS writes per stage.  The 4x2 kernels
    // need the registers (two waves per SIMD) and keep four producer waves that do both.
    constexpr int NPW = igemm_producer_waves(TM, TN, TAPS, UA, UB);
    constexpr bool SPLIT = NPW == 8;
    constexpr int THREADS = (NCW + NPW) * 64;
    constexpr int PTHREADS = NPW * 64;     // all producer threads (zero fill)
    constexpr int UTHREADS = 4 * 64;       // threads that share the units of one kind
    constexpr int KT = WN * TN * 32;       // filters per block   (MFMA B operand / D columns)
    constexpr int PT = WM * TM * 32;       // pixels per block    (MFMA A operand / D rows)
    constexpr int OCT = CC / 8;
    constexpr int KSTEPS = CC / 16;
    constexpr int PTP = PT + 8;            // pixel pitch of the staged output tile
    constexpr int WOP = igemm_filter_octet_pitch(KT, OCT);   // bytes between the octets of one tap in the filter region
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int BUF0 = 16;

    CVX_TRACE_MARK(0);
    warm_kernel_arguments<sizeof(ConvArgs) + sizeof(IgemmGeom)>();
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform by construction
    const bool producer = wave >= NCW;
#ifdef CVX_PHASE_TRACE
    if (lane == 0 && g_phase_trace) {
        // developer build: which SIMD each wave of the block landed on (HW_ID bits 5:4), 4 bits per wave
        const unsigned hw = __builtin_amdgcn_s_getreg((31 << 11) | 4);
        atomicOr(&g_phase_trace[((size_t)blockIdx.x + 2048) * 32], (unsigned long long)(((hw >> 4) & 3) + 1) << (4 * wave));
    }
#endif
    const int taps = TAPS > 0 ? TAPS : a.R * a.S;
    const int HW = a.H * a.W, HoWo = a.Ho * a.Wo;
    const int stage_bytes = g.xbytes + g.wbytes;

    // ---- which tile.  The hardware deals blocks round-robin over the 8 XCDs, each with its own L2.
    //      XCD x takes a rectangle of the (pixel block, filter block) grid, chosen on the host so that
    //      the chip fetches the least from device memory: every XCD reads the input of its pixel blocks
    //      and the filters of its filter blocks once.  Inside the rectangle, blocks that share an input
    //      tile (differing only in the filter block) are neighbours.
    int pb, kb;
    if (g.xcd_kparts > 0) {
        // the division constants of the rectangle come from the host: this decode is on the way to the
        // first load of every block
        const int x = blockIdx.x & 7, j = blockIdx.x >> 3;         // XCD, index inside it
        const int pbl = g.by_kpx.div(j);                           // j < 65536 here (host)
        pb = (x >> g.xcd_kshift) * g.xcd_ppx + pbl;
        kb = (x & (g.xcd_kparts - 1)) * (int)g.by_kpx.d + (j - pbl * (int)g.by_kpx.d);
    } else {
        const int kblocks = (int)g.by_kblocks.d;
        pb = kblocks == 1 ? (int)blockIdx.x : (int)blockIdx.x / kblocks;
        kb = (int)blockIdx.x - pb * kblocks;
    }
    const int rowblocks = (int)g.by_rowblocks.d;
    const int ib = rowblocks == 1 ? pb : (pb < 65536 ? g.by_rowblocks.div(pb) : pb / rowblocks);
    const int rb = pb - ib * rowblocks;
    // grouped convolution: filter block kb belongs to group grp, which reads input channels
    // [c_first, c_first + cg) and owns filters [k0 .. k_end)
    const int grp = g.kb_per_group == g.k_blocks ? 0 : kb / g.kb_per_group;
    const int k0 = grp * g.kg + (kb - grp * g.kb_per_group) * KT;
    const int k_end = (grp + 1) * g.kg;
    const int c_first = grp * g.cg;
    const int n0 = ib * g.NB;
    const int p0 = rb * g.TH;
    const int rows = min(g.TH, a.Ho - p0);
    const int nimg = min(g.NB, a.N - n0);
    const int ppi = rows * a.Wo;                       // output pixels per image in this tile
    const int npix = nimg * ppi;
    const int n_ptiles = (npix + 31) >> 5;             // pixel tiles holding at least one pixel

    if (producer) {
        // =========================================================================================
        // producer waves
        // =========================================================================================
        const int ptid = tid - NCW * 64;
        const bool input_wave = !SPLIT || wave < NCW + 4;          // wave-uniform role among the producers
        const bool filter_wave = !SPLIT || wave >= NCW + 4;
        const int utid = (SPLIT && !input_wave) ? ptid - UTHREADS : ptid;
        const long long x_total = (long long)a.N * a.C * HW;
        const long long w_total = (long long)a.K * g.cg * taps;
        const uint16_t* __restrict__ xg = (const uint16_t*)a.x;
        const uint16_t* __restrict__ wg = (const uint16_t*)a.w;
        const int h_lo = p0 * a.stride_h - a.pad_h;    // first input row of the patch (may be < 0)
        const int e_lo = h_lo * a.W;                   // flat element index of the patch start

        // What each thread fetches.  An input unit is 8 consecutive flat (h,w) elements of the patch
        // for the 8 channels of one octet.  A filter unit is (filter, octet): 8 channels x TAPS taps,
        // contiguous in memory.
        long long a_goff[UA];
        int a_oct[UA], a_img[UA], a_ui[UA];
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int ua = utid + u * UTHREADS;
            a_oct[u] = -1;
            a_goff[u] = 0;
            a_img[u] = 0;
            a_ui[u] = 0;
            if (input_wave && ua < g.a_units) {
                const int t = g.by_upi.div(ua);
                const int ui = ua - t * g.UPI;
                const int oct = g.by_nb.div(t);
                const int img = t - oct * g.NB;
                a_img[u] = img;
                a_ui[u] = ui;
                a_goff[u] = ((long long)(n0 + img) * a.C + c_first + oct * 8) * HW + e_lo + ui * 8;
                if (img < nimg) a_oct[u] = oct;        // images past N: nothing to fetch, LDS stays zero
            }
        }
        constexpr int BROWS = TAPS > 0 ? (8 * TAPS * 2 + 15) / 16 : 1;   // 16-byte loads per filter unit
        int b_k[UB], b_oct[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int ub = utid + u * UTHREADS;
            b_k[u] = ub / OCT;
            b_oct[u] = ub % OCT;
            if (!filter_wave || ub >= g.b_units) b_oct[u] = -1;
        }

        struct StageRegs {
            u32x4 ra[UA][8];
            u32x4 rbv[UB][BROWS];
        };
        StageRegs R0;

        // Global loads only; nothing here consumes a loaded value, so all of a stage's loads are in
        // flight together and are first waited on in store_stage.
        auto load_stage = [&](int st, StageRegs& R) {
            auto& ra = R.ra;
            auto& rbv = R.rbv;
            const int cbase = st * CC;
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                if (a_oct[u] >= 0) {
                    const int c0 = cbase + a_oct[u] * 8;
                    const long long off0 = a_goff[u] + (long long)cbase * HW;
                    const bool fast = off0 >= 0 && off0 + 7LL * HW + 8 <= x_total && c0 + 8 <= g.cg;
                    if (fast) {
#pragma unroll
                        for (int j = 0; j < 8; ++j) ra[u][j] = *(const u32x4_a2*)(xg + off0 + (long long)j * HW);
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            u32x4 v = {0u, 0u, 0u, 0u};
                            if (c0 + j < g.cg) v = load8(xg, off0 + (long long)j * HW, x_total);
                            ra[u][j] = v;
                        }
                    }
                }
            }
            if constexpr (TAPS > 0) {
#pragma unroll
                for (int u = 0; u < UB; ++u) {
                    if (b_oct[u] >= 0) {
                        const int k = k0 + b_k[u];
                        const int c0 = cbase + b_oct[u] * 8;
                        const long long off0 = ((long long)k * g.cg + c0) * TAPS;
                        const bool full = k < k_end && c0 + 8 <= g.cg;
                        if (full) {
#pragma unroll
                            for (int i = 0; i < BROWS; ++i) {
                                if (i * 8 + 8 <= 8 * TAPS) rbv[u][i] = *(const u32x4_a2*)(wg + off0 + i * 8);
                                else rbv[u][i] = load8(wg, off0 + i * 8, w_total);
                            }
                        } else {
                            // ragged: filters past K or channels past C contribute zeros
#pragma unroll
                            for (int i = 0; i < BROWS; ++i) {
                                u32x4 v = {0u, 0u, 0u, 0u};
#pragma unroll
                                for (int e = 0; e < 8; ++e) {
                                    const int t = i * 8 + e;          // = j * TAPS + tap
                                    const int j = t / TAPS;
                                    if (k < k_end && j < 8 && c0 + j < g.cg)
                                        v[e >> 1] |= ((uint32_t)wg[off0 + t]) << ((e & 1) * 16);
                                }
                                rbv[u][i] = v;
                            }
                        }
                    }
                }
            }
        };

        int a_dst[UA][8];
        auto prepare_lds = [&]() __attribute__((always_inline)) {
            // a_dst: the LDS byte offset (inside the input region) each of a unit's 8 elements goes to;
            // elements outside the image go to the region's trash slot.
#pragma unroll
            for (int u = 0; u < UA; ++u) {
#pragma unroll
                for (int e = 0; e < 8; ++e) a_dst[u][e] = g.xbytes - TRASH_BYTES + lane * 16;
                if (a_oct[u] >= 0) {
                    const int rel0 = a_ui[u] * 8;
                    int row = g.by_w.div(rel0);
                    int col = rel0 - row * a.W;
                    const int region = (a_oct[u] * g.NB + a_img[u]) * g.PSLOTS;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int eabs = e_lo + rel0 + e;
                        if (a_img[u] < nimg && eabs >= 0 && eabs < HW && row < g.PH)
                            a_dst[u][e] = (region + lds_slot(row * g.WP + col + a.pad_w)) * 16;
                        if (++col == a.W) { col = 0; ++row; }
                    }
                }
            }
            if (g.flat) {
                // where each pixel of the tile goes in the output staging (byte offset); pixels the tile does not
                // have go to a spare image region that is never copied out
                int* ftab = (int*)(smem + BUF0 + 2 * stage_bytes);
                for (int f = ptid; f < PT; f += PTHREADS) {
                    const int img = g.by_howo.div(f);
                    const int rem = f - img * HoWo;
                    const uint32_t sh = ((uint32_t)((n0 + img) * a.K + k0) * (uint32_t)HoWo) & 7u;
                    ftab[f] = f < npix ? (img * g.flat_pitch + (int)sh + rem) * 2 : (g.NB * g.flat_pitch + (f & 7)) * 2;
                }
            }
            {
                // zero both input regions: pad columns and rows outside the image are never written
                // afterwards, so they stay zero for every stage
                const u32x4 z = {0u, 0u, 0u, 0u};
                for (int i = ptid * 16; i < g.xbytes; i += PTHREADS * 16) {
                    *(u32x4*)(smem + BUF0 + i) = z;
                    *(u32x4*)(smem + BUF0 + stage_bytes + i) = z;
                }
            }
        };

        auto store_stage = [&](int st, int buf, const StageRegs& R) {
            auto& ra = R.ra;
            auto& rbv = R.rbv;
            unsigned char* xs = smem + BUF0 + buf * stage_bytes;
            unsigned char* ws = xs + g.xbytes;
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                if (a_oct[u] >= 0) {
                    // 8 channel rows x 8 elements  ->  8 elements x 8 channels
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        u32x4 o;
#pragma unroll
                        for (int m = 0; m < 4; ++m)
                            o[m] = pack_halves(ra[u][2 * m + 1][e >> 1], e & 1, ra[u][2 * m][e >> 1], e & 1);
                        *(u32x4*)(xs + a_dst[u][e]) = o;
                    }
                }
            }
            if constexpr (TAPS > 0) {
#pragma unroll
                for (int u = 0; u < UB; ++u) {
                    if (b_oct[u] >= 0) {
#pragma unroll
                        for (int tap = 0; tap < TAPS; ++tap) {
                            u32x4 o;
#pragma unroll
                            for (int m = 0; m < 4; ++m) {
                                const int t0 = (2 * m) * TAPS + tap, t1 = (2 * m + 1) * TAPS + tap;
                                o[m] = pack_halves(rbv[u][t1 >> 3][(t1 >> 1) & 3], t1 & 1,
                                                   rbv[u][t0 >> 3][(t0 >> 1) & 3], t0 & 1);
                            }
                            *(u32x4*)(ws + (tap * OCT + b_oct[u]) * WOP + b_k[u] * 16) = o;
                        }
                    }
                }
            } else {
                // any filter size: element-wise gather from global memory, scatter into LDS
                const int cbase = st * CC;
                for (int pi = filter_wave ? utid : KT * CC; pi < KT * CC; pi += UTHREADS) {
                    const int cl = pi % CC, kl = pi / CC;
                    const int k = k0 + kl, c = cbase + cl;
                    const bool ok = k < k_end && c < g.cg;
                    const long long off0 = ((long long)k * g.cg + c) * taps;
                    for (int t = 0; t < taps; ++t) {
                        const uint16_t v = ok ? wg[off0 + t] : (uint16_t)0;
                        *(uint16_t*)(ws + (t * OCT + (cl >> 3)) * WOP + kl * 16 + (cl & 7) * 2) = v;
                    }
                }
            }
        };

        // ---- the common case, with nothing conditional in it ---------------------------------------
        // The general loop above takes a different number of loads per stage depending on run-time
        // conditions (ragged channels or filters, offsets outside the tensor, lanes without a unit), so
        // the compiler cannot know how many loads are in flight behind the ones a stage needs and
        // waits for all of them: the second register set then buys nothing.  When every unit of every
        // stage of this wave is a plain in-bounds load, the loop below issues a fixed number of loads
        // per stage (lanes without a unit fetch a valid address and write nothing), and the waits become
        // "all but the newest stage" (c5b 50.0 -> 45.4 us).  Not for kernels with several units per
        // thread (no registers for two sets of them), and not for the twelve-wave kernels: their eight
        // producer waves already keep the memory pipeline full, and two stages of loads in flight per
        // wave measured slower (c5a 45.2 us against 43.9).
        constexpr bool FASTABLE = TAPS > 0 && UA == 1 && UB == 1 && !SPLIT;
        bool fast_lane = FASTABLE && (g.n_stages & 1) == 0 && g.cg % CC == 0 && k0 + KT <= k_end;
        long long w_goff[UB];
        int w_dst[UB];
        {
            const long long span = (long long)(g.n_stages - 1) * CC * HW + 7LL * HW + 8;
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                if (a_oct[u] < 0) a_goff[u] = ((long long)n0 * a.C + c_first) * HW + e_lo;
                if (input_wave) fast_lane = fast_lane && a_goff[u] >= 0 && a_goff[u] + span <= x_total;
            }
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int ub = utid + u * UTHREADS;
                const bool live = ub < g.b_units;
                const int k = live ? ub / OCT : 0, oct = live ? ub % OCT : 0;
                w_goff[u] = ((long long)(k0 + k) * g.cg + oct * 8) * (TAPS > 0 ? TAPS : 1);
                w_dst[u] = live ? oct * WOP + k * 16 : -1;
            }
        }
        const bool fast_wave = __builtin_amdgcn_ballot_w64(!fast_lane) == 0ull;

        auto run_fast = [&]() __attribute__((always_inline)) {
            constexpr bool DO_X = true, DO_W = true;
            u32x4 xa[2][UA][8];
            u32x4 wb[2][UB][BROWS];
            const int last = g.n_stages - 1;
            auto load = [&](int st, auto set_c) __attribute__((always_inline)) {
                constexpr int SET = decltype(set_c)::value;
                // past the last stage the same number of loads is issued, all lanes at the start of the
                // tensor (one cache line; the values are never used)
                const bool real = st <= last;
                const int cbase = st * CC;
                if constexpr (DO_X) {
#pragma unroll
                    for (int u = 0; u < UA; ++u) {
                        const uint16_t* p = real ? xg + a_goff[u] + (long long)cbase * HW : xg;
#pragma unroll
                        for (int j = 0; j < 8; ++j) xa[SET][u][j] = *(const u32x4_a2*)(p + (long long)j * HW);
                    }
                }
                if constexpr (DO_W) {
#pragma unroll
                    for (int u = 0; u < UB; ++u) {
                        const uint16_t* p = real ? wg + w_goff[u] + (long long)cbase * TAPS : wg;
#pragma unroll
                        for (int i = 0; i < BROWS; ++i) wb[SET][u][i] = *(const u32x4_a2*)(p + i * 8);
                    }
                }
            };
            // One half-iteration: transpose register set SET (stage s) into temporaries, refill the set
            // with the loads of stage s+2 right away (the transposed copy is what gets written), then
            // write the temporaries into LDS buffer `buf`.  Lanes without a unit skip only the writes.
            auto step = [&](int buf, auto set_c, int st_next, auto refill_c) __attribute__((always_inline)) {
                constexpr int SET = decltype(set_c)::value;
                constexpr bool REFILL = decltype(refill_c)::value;
                unsigned char* xs = smem + BUF0 + buf * stage_bytes;
                const bool real = st_next <= last;
                const int cbase = st_next * CC;
                if constexpr (DO_X) {
#pragma unroll
                    for (int u = 0; u < UA; ++u) {
                        u32x4 o[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e)
#pragma unroll
                            for (int m = 0; m < 4; ++m)
                                o[e][m] = pack_halves(xa[SET][u][2 * m + 1][e >> 1], e & 1, xa[SET][u][2 * m][e >> 1], e & 1);
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (REFILL) {
                            const uint16_t* p = real ? xg + a_goff[u] + (long long)cbase * HW : xg;
#pragma unroll
                            for (int j = 0; j < 8; ++j) xa[SET][u][j] = *(const u32x4_a2*)(p + (long long)j * HW);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        if (a_oct[u] >= 0) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) *(u32x4*)(xs + a_dst[u][e]) = o[e];
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if constexpr (DO_W) {
                    unsigned char* ws = xs + g.xbytes;
#pragma unroll
                    for (int u = 0; u < UB; ++u) {
                        u32x4 o[TAPS > 0 ? TAPS : 1];
#pragma unroll
                        for (int tap = 0; tap < TAPS; ++tap)
#pragma unroll
                            for (int m = 0; m < 4; ++m) {
                                const int t0 = (2 * m) * TAPS + tap, t1 = (2 * m + 1) * TAPS + tap;
                                o[tap][m] = pack_halves(wb[SET][u][t1 >> 3][(t1 >> 1) & 3], t1 & 1,
                                                        wb[SET][u][t0 >> 3][(t0 >> 1) & 3], t0 & 1);
                            }
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (REFILL) {
                            const uint16_t* p = real ? wg + w_goff[u] + (long long)cbase * TAPS : wg;
#pragma unroll
                            for (int i = 0; i < BROWS; ++i) wb[SET][u][i] = *(const u32x4_a2*)(p + i * 8);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        if (w_dst[u] >= 0) {
#pragma unroll
                            for (int tap = 0; tap < TAPS; ++tap) *(u32x4*)(ws + tap * OCT * WOP + w_dst[u]) = o[tap];
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            };
            const std::integral_constant<int, 0> s0;
            const std::integral_constant<int, 1> s1;
            load(0, s0);
            load(1, s1);
            prepare_lds();
            __syncthreads();                           // (A) zero fill complete
            const std::true_type refill;
            step(0, s0, 2, refill);                    // stage 0 into LDS, stage 2 into its registers
            __syncthreads();                           // (B) stage 0 is in LDS
            for (int st = 0; st + 2 < g.n_stages; st += 2) {
                step(1, s1, st + 3, refill);           // stage st+1
                __syncthreads();                       // stage st consumed, stage st+1 in LDS
                step(0, s0, st + 4, refill);           // stage st+2
                __syncthreads();                       // stage st+1 consumed, stage st+2 in LDS
            }
            step(1, s1, 0, std::false_type());         // the last stage; nothing follows it
            __syncthreads();
            __syncthreads();                           // the consumers' barrier after the last stage
        };

        if (FASTABLE && fast_wave) {
            run_fast();
        } else {
            // general loop (ragged tiles, tensor edges, odd stage counts, filter sizes without a compiled
            // transpose): one register set; the loads of stage st+2 are issued once stage st+1 has been
            // transposed out of it
            load_stage(0, R0);
            prepare_lds();
            __syncthreads();                               // (A) zero fill complete
            store_stage(0, 0, R0);
            if (g.n_stages > 1) load_stage(1, R0);
            __syncthreads();                               // (B) stage 0 is in LDS
            CVX_TRACE_MARK_T(2, NCW * 64);
            for (int st = 0; st < g.n_stages; ++st) {
                if (st + 1 < g.n_stages) {
                    store_stage(st + 1, (st + 1) & 1, R0);
                    if (st + 2 < g.n_stages) load_stage(st + 2, R0);
                }
                if (st < 6) CVX_TRACE_MARK_T(4 + 2 * st, NCW * 64);
                __syncthreads();                           // stage st consumed, stage st+1 in LDS
            }
        }
    } else {
        // =========================================================================================
        // consumer waves
        // =========================================================================================
        const int l32 = lane & 31, half = lane >> 5;
        const int wm = wave / WN, wn = wave % WN;

        // Per-lane LDS byte offsets for each of the wave's pixel tiles: xb[tm][s] addresses filter
        // column s of filter row 0 (octet `half`); further filter rows are a constant row_bytes away.
        // Kernels built for a fixed filter size keep one offset per filter column; the others keep the
        // logical element index and derive the address per tap.
        constexpr int NSW = TAPS == 9 ? 3 : 1;
        const int oct_bytes = g.NB * g.PSLOTS * 16;
        const int row_bytes = a.dil_h * g.WP * 18;                 // one filter row down, in bytes
        int xb[TM][NSW];
        int xl[TM], xr[TM];                                        // logical element, region byte offset
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int f = (tm * WM + wm) * 32 + l32;      // pixel tiles are dealt round-robin to the wave rows
            int img = 0, rem = f;
            if (g.NB > 1) {                 // multi-image tiles hold whole images: ppi = Ho * Wo
                img = f / ppi;
                rem = f - img * ppi;
            }
            const int py = g.by_wo.div(rem);
            const int px = rem - py * a.Wo;
            const bool valid = f < npix;
            // Rows of a tile past the block's pixels still go through the matrix pipe.  They are pointed at
            // zeros where the layout has them -- the columns after the image's last one (right padding, the
            // spare columns of the rounded pitch, the next row's left padding) -- because the chip runs at
            // its power limit and multiplying zeros costs less of it than multiplying whatever sits at
            // element 0.
            const int zero_col = (g.WP - a.W >= (a.S - 1) * a.dil_w + 1) ? a.W + a.pad_w : 0;
            xl[tm] = valid ? py * a.stride_h * g.WP + px * a.stride_w : zero_col;
            xr[tm] = (valid ? img * g.PSLOTS * 16 : 0) + half * oct_bytes;
#pragma unroll
            for (int sw = 0; sw < NSW; ++sw) xb[tm][sw] = xr[tm] + lds_slot(xl[tm] + sw * a.dil_w) * 16;
        }
        const int b_lane = ((wn * TN) * 32 + l32) * 16 + half * WOP;
        const bool wave_on = wm < n_ptiles;            // this wave owns at least one live pixel tile

        // epilogue constants of this lane's filters: only the loads are issued here; they are turned
        // into (mul, add) after the prologue barriers, when they have long arrived
        const bool has_bn = a.bn_scale != nullptr;
        uint32_t bias_raw[TN];
        float bn_raw[TN][4];
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int k = min(k0 + (wn * TN + tn) * 32 + l32, a.K - 1);
            bias_raw[tn] = 0u;
            if (a.bias) bias_raw[tn] = a.bias_f32 ? ((const uint32_t*)a.bias)[k] : (uint32_t)((const uint16_t*)a.bias)[k];
#pragma unroll
            for (int j = 0; j < 4; ++j) bn_raw[tn][j] = 0.0f;
            if (has_bn) {
                bn_raw[tn][0] = a.bn_scale[k];
                bn_raw[tn][1] = a.bn_shift[k];
                bn_raw[tn][2] = a.bn_mean[k];
                bn_raw[tn][3] = a.bn_var[k];
            }
        }
        ChannelAffine ca[TN];

        f32x16 acc[TM][TN];

        // One k-step = one filter tap x 16 channels: TM pixel fragments (MFMA A operand), TN filter
        // fragments (B operand), TM*TN MFMAs.  The instruction order is pinned: after each of the
        // first TM+TN MFMAs of a step, one fragment of the NEXT step is read (filters first, then
        // pixels in the order the MFMAs will want them), so LDS latency hides behind the matrix pipe
        // and the waits the compiler inserts are partial.
        // The consumer loop of the compiled filter sizes.  This wave is the only one on its SIMD that feeds
        // the matrix pipe, so whatever it issues between two MFMAs besides LDS reads is paid for in
        // matrix-pipe time: an address add that the next read has to wait for, a branch around an MFMA.
        // Hence: no branches in the loop; the filter fragments hang off one address register (wa) by
        // immediate offsets; and the addresses of a k-step's pixel fragments are computed a whole k-step
        // before their reads are issued (one add each, nothing waits for it).
        const int lds0 = (int)(uintptr_t)(lds_ptr_t)smem;          // LDS byte address of the dynamic allocation
        auto lds_read128 = [](int addr) __attribute__((always_inline)) {
            return *(const __attribute__((address_space(3))) u32x4*)(uintptr_t)(uint32_t)addr;
        };
        int wa = lds0 + (int)(BUF0 + g.xbytes + b_lane);
        auto compute_stage = [&](int buf) {
            if (!wave_on) return;
            const unsigned char* xs = smem + BUF0 + buf * stage_bytes;
            const unsigned char* ws = xs + g.xbytes + b_lane;
            if constexpr (TAPS == 9 || TAPS == 1) {
                constexpr int NS = TAPS * KSTEPS;
                const int xs_off = lds0 + BUF0 + buf * stage_bytes;
                // Fragments are read PF k-steps ahead of their MFMAs.  A step of 2x2 tiles is only
                // 4 MFMAs (128 clocks), shorter than the LDS latency under load, so those variants look
                // two steps ahead (three register sets); 4x2 tiles cover the latency with one.
                constexpr int PF = (TM * TN <= 4 && NS >= 3) ? 2 : 1;
                constexpr int NSET = PF + 1;
                constexpr bool SKIP_DEAD_TILES = TM * TN >= 8;
                const bool last_tile_live = (TM - 1) * WM + wm < n_ptiles;
                u32x4 fa[NSET][TM], fb[NSET][TN];
                int pa[TM];                                       // addresses of the pixel fragments of one k-step
                auto pixel_addresses = [&](int step) {
                    const int tap = step / KSTEPS, kk = step % KSTEPS;
                    const int soff = xs_off + (TAPS == 9 ? tap / 3 : 0) * row_bytes + 2 * kk * oct_bytes;   // wave-uniform
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) {
                        pa[tm] = xb[tm][TAPS == 9 ? tap % 3 : 0] + soff;
                        asm volatile("" : "+v"(pa[tm]));           // computed here, not where it is used
                    }
                };
                auto read_frag = [&](int set, int step, int which) {   // which: 0..TN-1 filters, TN.. pixels
                    const int tap = step / KSTEPS, kk = step % KSTEPS;
                    if (which < TN) fb[set][which] = lds_read128(wa + ((tap * OCT + 2 * kk) * WOP + which * 32 * 16));
                    else fa[set][which - TN] = lds_read128(pa[which - TN]);
                };
#pragma unroll
                for (int p = 0; p < PF; ++p) {
                    pixel_addresses(p);
#pragma unroll
                    for (int j = 0; j < TM + TN; ++j) read_frag(p, p, j);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < NS; ++i) {
                    const int cur = i % NSET, nxt = (i + PF) % NSET;
                    const bool more = i + PF < NS;
                    int issued = 0;
                    if (more) {
                        pixel_addresses(i + PF);
                        __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) {
                        // A pixel tile past the end of the block's pixels (wave-uniform; only a wave's last
                        // tile can be one) costs no matrix work and no operand traffic: c5b, where 196 of 256
                        // pixel rows are live, 43.9 -> 40.0 us.  One branch per tile and k-step, not per MFMA;
                        // the 2x2 kernels do without (there the branches cost what the spared MFMAs save).
                        // (both branches issue the same reads, so what has been issued stays a compile-time fact)
                        const bool dead = SKIP_DEAD_TILES && tm == TM - 1 && !last_tile_live;
                        const int first = issued;
                        if (!dead) {
#pragma unroll
                            for (int tn = 0; tn < TN; ++tn) {
                                acc[tm][tn] = mfma_32x32x16<DT>(fa[cur][tm], fb[cur][tn], acc[tm][tn]);
                                __builtin_amdgcn_sched_barrier(0);
                                if (more && first + tn < TM + TN) {
                                    read_frag(nxt, i + PF, first + tn);
                                    __builtin_amdgcn_sched_barrier(0);
                                }
                            }
                        } else {
#pragma unroll
                            for (int tn = 0; tn < TN; ++tn) {
                                if (more && first + tn < TM + TN) {
                                    read_frag(nxt, i + PF, first + tn);
                                    __builtin_amdgcn_sched_barrier(0);
                                }
                            }
                        }
                        issued = first + TN < TM + TN ? first + TN : TM + TN;
                    }
#pragma unroll
                    for (int j = 0; j < TM + TN; ++j) {
                        if (more && issued < TM + TN) {
                            read_frag(nxt, i + PF, issued);
                            ++issued;
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                }
                wa += buf ? -stage_bytes : stage_bytes;
            } else {
                int r = 0, s = 0;
                for (int tap = 0; tap < taps; ++tap) {
                    int ta[TM];
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) ta[tm] = xr[tm] + lds_slot(xl[tm] + s * a.dil_w) * 16 + r * row_bytes;
#pragma unroll
                    for (int kk = 0; kk < KSTEPS; ++kk) {
                        u32x4 fa[TM], fb[TN];
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn) fb[tn] = *(const u32x4*)(ws + (tap * OCT + 2 * kk) * WOP + tn * 32 * 16);
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm) fa[tm] = *(const u32x4*)(xs + ta[tm] + 2 * kk * oct_bytes);
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                            for (int tn = 0; tn < TN; ++tn) acc[tm][tn] = mfma_32x32x16<DT>(fa[tm], fb[tn], acc[tm][tn]);
                    }
                    if (++s == a.S) { s = 0; ++r; }
                }
            }
        };

        CVX_TRACE_MARK(1);
        __syncthreads();                               // (A)
        __syncthreads();                               // (B) stage 0 is in LDS
        // the bias loads issued above have had the whole prologue to arrive; without batch-norm the
        // bias seeds the accumulators
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            float b = 0.0f;
            if (a.bias) b = a.bias_f32 ? __uint_as_float(bias_raw[tn]) : bits16_to_f32<DT>((uint16_t)bias_raw[tn]);
            if (has_bn) {
                const float m = bn_raw[tn][0] / sqrtf(bn_raw[tn][3] + a.bn_eps);
                ca[tn].mul = m;
                ca[tn].add = (b - bn_raw[tn][2]) * m + bn_raw[tn][1];
            } else {
                ca[tn].mul = 1.0f;
                ca[tn].add = b;
            }
        }
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const float seed = has_bn ? 0.0f : ca[tn].add;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[tm][tn][r] = seed;
            }
#ifdef CVX_PHASE_TRACE
        long long tr_mul = 0, tr_bar = 0, tr_first = 0;      // developer build: shader clocks spent multiplying / at the barrier
#endif
        for (int st = 0; st < g.n_stages; ++st) {
#ifdef CVX_PHASE_TRACE
            const long long tq0 = clock64();
#endif
            compute_stage(st & 1);
            if (st < 6) CVX_TRACE_MARK(3 + 2 * st);
#ifdef CVX_PHASE_TRACE
            const long long tq1 = clock64();
#endif
            __syncthreads();
#ifdef CVX_PHASE_TRACE
            tr_mul += tq1 - tq0;
            tr_bar += clock64() - tq1;
            if (st == 0) tr_first = tq1 - tq0;
#endif
        }
        CVX_TRACE_MARK(14);
#ifdef CVX_PHASE_TRACE
        if (threadIdx.x == 0 && g_phase_trace) {
            g_phase_trace[(size_t)blockIdx.x * 32 + 16 + 10] = tr_mul;
            g_phase_trace[(size_t)blockIdx.x * 32 + 16 + 11] = tr_bar;
            g_phase_trace[(size_t)blockIdx.x * 32 + 16 + 12] = tr_first;
        }
#endif

        // ---- epilogue, part 1: batch-norm / activation on the accumulators in registers, one
        //      rounding to the output type, then the tile goes into LDS as [filter][pixel].
        // Two stagings.  Ordinarily the tile is [filter][pixel] and the store below walks along the
        // pixel axis.  For tiles of whole images whose planes are not a multiple of 16 bytes (7x7, 14x14
        // images) a filter row starts at any 2-byte offset of y and 8-pixel pieces straddle images; but
        // the planes of the block's filters follow each other in y, so per image the block owns one
        // contiguous run of y, and the tile is staged as exactly that run, shifted so that 16-byte
        // pieces of LDS are aligned 16-byte pieces of y.  The store is then a plain copy.  Where each
        // pixel goes comes from a table the producers wrote in the prologue.
        uint16_t* ot = (uint16_t*)(smem + BUF0);
        if (wave_on) {
            const int* ftab = (const int*)(smem + BUF0 + 2 * stage_bytes);
            // Runs of y: a lane's four consecutive pixels stay together when the planes are multiples of
            // 4 pixels; otherwise every pixel has its own place.
            const bool by_pixel = g.flat == 1;
            auto stage_out = [&](auto&& convert) __attribute__((always_inline)) {
                if (g.flat == 0) {
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        const int kl = (wn * TN + tn) * 32 + l32;
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                            for (int q4 = 0; q4 < 4; ++q4) {
                                uint32_t p0, p1;
                                convert(acc[tm][tn], tn, q4, p0, p1);
                                const int f = (tm * WM + wm) * 32 + 8 * q4 + 4 * half;
                                *(uint2*)(ot + kl * PTP + f) = make_uint2(p0, p1);
                            }
                    }
                    return;
                }
                int krow[TN];
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) krow[tn] = ((wn * TN + tn) * 32 + l32) * HoWo * 2;
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    const int f0 = (tm * WM + wm) * 32 + 4 * half;
                    if (!by_pixel) {
                        int fo[4];
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) fo[q4] = ftab[f0 + 8 * q4];
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                            for (int tn = 0; tn < TN; ++tn) {
                                uint32_t p0, p1;
                                convert(acc[tm][tn], tn, q4, p0, p1);
                                *(uint2*)((unsigned char*)ot + fo[q4] + krow[tn]) = make_uint2(p0, p1);
                            }
                    } else {
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            const int4 t = *(const int4*)(ftab + f0 + 8 * q4);
#pragma unroll
                            for (int tn = 0; tn < TN; ++tn) {
                                uint32_t p0, p1;
                                convert(acc[tm][tn], tn, q4, p0, p1);
                                unsigned char* o = (unsigned char*)ot + krow[tn];
                                *(uint16_t*)(o + t.x) = (uint16_t)p0;
                                *(uint16_t*)(o + t.y) = (uint16_t)(p0 >> 16);
                                *(uint16_t*)(o + t.z) = (uint16_t)p1;
                                *(uint16_t*)(o + t.w) = (uint16_t)(p1 >> 16);
                            }
                        }
                    }
                }
            };
            auto with_act = [&](auto&& act_fn) __attribute__((always_inline)) {
                stage_out([&](const f32x16& t, int tn, int q4, uint32_t& p0, uint32_t& p1) __attribute__((always_inline)) {
                    float v[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = act_fn(has_bn ? fmaf(t[4 * q4 + j], ca[tn].mul, ca[tn].add) : t[4 * q4 + j]);
                    p0 = pack2<DT>(v[0], v[1]);
                    p1 = pack2<DT>(v[2], v[3]);
                });
            };
            if ((a.act == ACT_RELU || a.act == ACT_IDENTITY) && !has_bn) {
                // the common case (the bias is already in the accumulators), kept short because only the
                // consumer waves can do it: round, then ReLU on the packed pair, 1 instruction per value
                const uint32_t floor2 = packed_floor(a.act == ACT_RELU);
                stage_out([&](const f32x16& t, int, int q4, uint32_t& p0, uint32_t& p1) __attribute__((always_inline)) {
                    p0 = max_packed(pack2<DT>(t[4 * q4], t[4 * q4 + 1]), floor2);
                    p1 = max_packed(pack2<DT>(t[4 * q4 + 2], t[4 * q4 + 3]), floor2);
                });
            } else if (a.act == ACT_RELU) with_act([](float t) { return fmaxf(t, 0.0f); });
            else if (a.act == ACT_IDENTITY) with_act([](float t) { return t; });
            else with_act([&](float t) { return activate(t, a.act, a.alpha); });
        }
    }
    __syncthreads();                                   // output tile complete in LDS

    // ---- epilogue, part 2 (all waves): the single store to device memory, 16 bytes per lane along
    //      the pixel axis.
    if (g.flat) {
        // the staged runs are copied out: 16 aligned bytes per lane, consecutive lanes consecutive pieces
        const unsigned char* ot = smem + BUF0;
        uint16_t* __restrict__ yg = (uint16_t*)a.y;
        const int len = min(KT, k_end - k0) * HoWo;                 // elements of one image's run
        for (int img = 0; img < nimg; ++img) {
            const size_t e0 = ((size_t)(n0 + img) * a.K + k0) * HoWo;   // first element of the run in y
            const int sh = (int)(e0 & 7);
            const int nch = (len + sh + 7) >> 3;
            uint16_t* dst0 = yg + (e0 - sh);                        // 16-byte aligned: y itself is
            const unsigned char* src = ot + (size_t)img * g.flat_pitch * 2;
            for (int c = tid; c < nch; c += THREADS) {
                const u32x4 v = *(const u32x4*)(src + c * 16);
                if (8 * c >= sh && 8 * c + 8 <= sh + len) {
                    __builtin_nontemporal_store(v, (u32x4*)(dst0 + 8 * c));
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (8 * c + e >= sh && 8 * c + e < sh + len) dst0[8 * c + e] = (uint16_t)(v[e >> 1] >> ((e & 1) * 16));
                }
            }
        }
    } else {
        const uint16_t* ot = (const uint16_t*)(smem + BUF0);
        constexpr int CH = PT / 8;                 // 8-pixel chunks per filter row
        constexpr int RSTEP = THREADS / CH;        // filter rows covered per pass
        constexpr int NPASS = (KT + RSTEP - 1) / RSTEP;
        const int chunk = tid % CH, row0 = tid / CH;
        const int f0 = chunk * 8;
        if (f0 < npix) {
            int img = 0, rem = f0;
            if (g.NB > 1) {
                img = f0 / ppi;
                rem = f0 - img * ppi;
            }
            const bool whole = rem + 8 <= ppi;     // all 8 pixels valid and inside one image
            uint16_t* __restrict__ yg = (uint16_t*)a.y;
            const size_t obase = ((size_t)(n0 + img) * a.K + k0) * HoWo + (size_t)p0 * a.Wo + rem;
            // A chunk that straddles an image boundary or the end of the tile is stored element by
            // element; where each element goes (relative to the chunk's first) is the same for every
            // filter row, so it is worked out once, by stepping, not by dividing: -1 = past the tile.
            int eoff[8];
            if (!whole) {
                int r = rem, jump = 0;                 // jump: offset of the current image relative to the first
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if (r == ppi) {                    // next image of the tile: K * HoWo further, back at its first pixel
                        r = 0;
                        jump += a.K * HoWo - ppi;
                    }
                    eoff[e] = f0 + e < npix ? e + jump : -1;
                    ++r;
                }
            }
            const bool tail4 = !whole && f0 + 4 == npix && rem + 4 <= ppi;   // four live pixels, all in one image
            constexpr int GRP = NPASS >= 4 ? 4 : NPASS;
            for (int p = 0; p < NPASS; p += GRP) {
                u32x4 v[GRP];
#pragma unroll
                for (int j = 0; j < GRP; ++j) {
                    const int kl = min(row0 + (p + j) * RSTEP, KT - 1);
                    v[j] = *(const u32x4*)(ot + kl * PTP + f0);
                }
#pragma unroll
                for (int j = 0; j < GRP; ++j) {
                    const int kl = row0 + (p + j) * RSTEP;
                    if (kl < KT && k0 + kl < k_end) {
                        uint16_t* dst = yg + obase + (size_t)kl * HoWo;
                        if (whole) {
                            // streaming store: lines left dirty in L2 would have to be written back at the end of the kernel
                            __builtin_nontemporal_store(v[j], (u32x4_a2*)dst);
                        } else {
                            // chunk straddles an image boundary or the end of the tile: element-wise
                            if (tail4 && (((uintptr_t)dst) & 7) == 0) {
                                // the tile ends after this chunk's first four pixels: one 8-byte store
                                *(uint2*)dst = make_uint2(v[j][0], v[j][1]);
                            } else {
#pragma unroll
                                for (int e = 0; e < 8; ++e)
                                    if (eoff[e] >= 0) dst[eoff[e]] = (uint16_t)(v[j][e >> 1] >> ((e & 1) * 16));
                            }
                        }
                    }
                }
            }
        }
    }
    CVX_TRACE_MARK(15);
}

// ------------------------------------------------------------------------------------------------
// host side: tile geometry, variant table, launch
// ------------------------------------------------------------------------------------------------
namespace {

constexpr int LDS_LIMIT = 160 * 1024;

struct Variant {
    const char* name;
    int WM, WN, TM, TN, CC, TAPS, UA, UB;     // waves / tiles along pixels (M) and filters (N)
    void (*kern_bf16)(ConvArgs, IgemmGeom);
    void (*kern_f16)(ConvArgs, IgemmGeom);
};

#define IGEMM_VARIANT(nm, WM, WN, TM, TN, CC, TAPS, UA, UB)                                          \
    {nm, WM, WN, TM, TN, CC, TAPS, UA, UB, igemm_kernel<DT_BF16, WM, WN, TM, TN, CC, TAPS, UA, UB>, \
     igemm_kernel<DT_F16, WM, WN, TM, TN, CC, TAPS, UA, UB>}

// name: igemm_<pixels per block>x<filters per block>_c<channels per stage>_<taps>
const Variant kVariants[] = {
    IGEMM_VARIANT("igemm_512x64_c32_3x3", 4, 1, 4, 2, 32, 9, 1, 1),
    IGEMM_VARIANT("igemm_512x64_c16_3x3", 4, 1, 4, 2, 16, 9, 1, 1),
    IGEMM_VARIANT("igemm_256x128_c16_3x3", 4, 1, 2, 4, 16, 9, 1, 1),
    IGEMM_VARIANT("igemm_256x64_c32_3x3", 4, 1, 2, 2, 32, 9, 1, 1),
    IGEMM_VARIANT("igemm_256x64_c16_3x3", 4, 1, 2, 2, 16, 9, 1, 1),
    IGEMM_VARIANT("igemm_256x64_c16_3x3_u2", 4, 1, 2, 2, 16, 9, 2, 1),
    IGEMM_VARIANT("igemm_128x128_c32_3x3", 2, 2, 2, 2, 32, 9, 1, 2),
    IGEMM_VARIANT("igemm_512x64_c32_1x1", 4, 1, 4, 2, 32, 1, 1, 1),
    IGEMM_VARIANT("igemm_512x64_c64_1x1", 4, 1, 4, 2, 64, 1, 2, 2),
    IGEMM_VARIANT("igemm_256x64_c32_1x1", 4, 1, 2, 2, 32, 1, 1, 1),
    IGEMM_VARIANT("igemm_256x64_c64_1x1", 4, 1, 2, 2, 64, 1, 1, 2),
    IGEMM_VARIANT("igemm_128x128_c64_1x1", 2, 2, 2, 2, 64, 1, 1, 4),
    IGEMM_VARIANT("igemm_256x64_c16_any", 4, 1, 2, 2, 16, 0, 2, 1),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

FastDiv fast_div(int d)
{
    FastDiv f;
    f.d = (uint32_t)d;
    f.m = d > 1 ? (uint32_t)(((1ull << 32) + (uint32_t)d - 1) / (uint32_t)d) : 0u;
    return f;
}

int lds_bytes(const Variant& v, const IgemmGeom& g)
{
    const int KT = v.WN * v.TN * 32, PT = v.WM * v.TM * 32;
    const int stages = 16 + 2 * (g.xbytes + g.wbytes) + (g.flat ? PT * 4 : 0);   // + the table of staging offsets
    const int otile = 16 + (g.flat ? (g.NB + 1) * g.flat_pitch * 2 : KT * (PT + 8) * 2);
    return stages > otile ? stages : otile;
}

// Tile geometry for a variant with a given pixel-tile shape (NB images x TH output rows, full
// width); returns false if the problem does not fit the variant that way.
bool plan(const ConvArgs& a, const Variant& v, int NB, int TH, IgemmGeom* out)
{
    const int taps = a.R * a.S;
    if (v.TAPS > 0 && v.TAPS != taps) return false;
    if (v.TAPS == 9 && (a.R != 3 || a.S != 3)) return false;      // the 9-tap kernels index taps as 3 x 3
    const int threads = 4 * 64;                    // producer threads
    const int KT = v.WN * v.TN * 32, PT = v.WM * v.TM * 32, OCT = v.CC / 8;
    if (NB < 1 || TH < 1 || NB > a.N || TH > a.Ho) return false;
    if (NB > 1 && TH != a.Ho) return false;
    if ((long long)NB * TH * a.Wo > PT) return false;
    if (a.W >= 32768 || a.Wo >= 32768) return false;
    IgemmGeom g;
    memset(&g, 0, sizeof g);
    g.NB = NB;
    g.TH = TH;
    g.PH = (g.TH - 1) * a.stride_h + (a.R - 1) * a.dil_h + 1;
    g.WP = (a.W + 2 * a.pad_w + 7) & ~7;
    const long long slots = (long long)g.PH * g.WP;
    const long long upi = ((long long)g.PH * a.W + 7) / 8;
    if (slots > 65535 || upi > 65535) return false;
    g.UPI = (int)upi;
    g.SLOTS = (int)slots;
    g.PSLOTS = g.SLOTS + g.SLOTS / 8 + 1;
    g.row_blocks = (a.Ho + g.TH - 1) / g.TH;
    g.img_blocks = (a.N + g.NB - 1) / g.NB;
    g.cg = a.C / a.groups;
    g.kg = a.K / a.groups;
    g.kb_per_group = (g.kg + KT - 1) / KT;
    g.k_blocks = g.kb_per_group * a.groups;
    g.n_stages = (g.cg + v.CC - 1) / v.CC;
    const long long a_units = (long long)OCT * g.NB * g.UPI;
    if (a_units > (long long)v.UA * threads) return false;
    g.a_units = (int)a_units;
    g.b_units = v.TAPS > 0 ? KT * OCT : 0;
    if (g.b_units > v.UB * threads) return false;
    const long long xb = (long long)OCT * g.NB * g.PSLOTS * 16 + TRASH_BYTES, wb = (long long)taps * OCT * igemm_filter_octet_pitch(KT, OCT);
    if (16 + 2 * (xb + wb) > LDS_LIMIT) return false;
    g.xbytes = (int)xb;
    g.wbytes = (int)wb;
    {
        // whole-image tiles with planes that are not a multiple of 16 bytes are staged as runs of y,
        // if that staging fits where the stage buffers were (else the ordinary tile is used)
        const int HoWo = a.Ho * a.Wo;
        if (TH == a.Ho && (HoWo & 7) != 0) {
            g.flat = (HoWo & 3) == 0 ? 2 : 1;
            g.flat_pitch = (KT * HoWo + 7 + 7) & ~7;
            if ((long long)(NB + 1) * g.flat_pitch * 2 > 2 * (xb + wb) || lds_bytes(v, g) > LDS_LIMIT) g.flat = 0;
        }
    }
    if (lds_bytes(v, g) > LDS_LIMIT) return false;
    if ((long long)g.row_blocks * g.img_blocks * g.k_blocks > 0x7fffffffLL) return false;
    g.by_wo = fast_div(a.Wo);
    g.by_w = fast_div(a.W);
    g.by_upi = fast_div(g.UPI);
    g.by_nb = fast_div(g.NB);
    // XCD rectangles: p pixel-block ranges x k filter-block ranges, p * k = 8; the chip then fetches about
    // k * input + p * filters bytes (each XCD its ranges once)
    g.xcd_kparts = 0;
    {
        const long long pblocks = (long long)g.row_blocks * g.img_blocks, nblk = pblocks * g.k_blocks;
        const double in_bytes = 2.0 * a.N * a.C * a.H * a.W, w_bytes = 2.0 * a.K * g.cg * taps;
        double best = 1e300;
        // (the in-kernel decode divides the index inside an XCD with a 16-bit magic number)
        for (int k = 1, sh = 0; k <= 8 && (nblk & 7) == 0 && (nblk >> 3) < 65536; k *= 2, ++sh) {
            const int pp = 8 / k;
            if (g.k_blocks % k || pblocks % pp) continue;
            const double fetched = k * in_bytes + pp * w_bytes;
            if (fetched < best) {
                best = fetched;
                g.xcd_kparts = k;
                g.xcd_kshift = sh;
                g.xcd_ppx = (int)(pblocks / pp);
                g.by_kpx = fast_div(g.k_blocks / k);
            }
        }
    }
    g.by_kblocks = fast_div(g.k_blocks);
    g.by_rowblocks = fast_div(g.row_blocks);
    g.by_howo = fast_div(a.Ho * a.Wo);
    *out = g;
    return true;
}

// Relative time estimate in MFMA-clock cycles: rounds of blocks over the compute units, each round
// costing the busiest wave's MFMA time plus a fixed fill/drain overhead, plus the bytes staged
// through LDS (halo and filter re-reads) at a nominal rate.
double cost(const ConvArgs& a, const Variant& v, const IgemmGeom& g, int cus)
{
    const long long blocks = (long long)g.row_blocks * g.img_blocks * g.k_blocks;
    const long long rounds = (blocks + cus - 1) / cus;
    const int used = (g.NB * g.TH * a.Wo + 31) / 32;
    // every wave multiplies all TM of its tiles (dead ones included) unless it has none at all
    const int per_wave = used >= 1 ? v.TM : 0;
    const double mfma = 32.0 * per_wave * v.TN * (a.R * a.S) * (v.CC / 16) * g.n_stages;
    // fixed launch/drain cost, a barrier hand-over per stage, and the fill of the first stage (which
    // nothing overlaps): smaller stages start the matrix pipe sooner
    const double overhead = 3000.0 + 400.0 * g.n_stages + (g.xbytes + g.wbytes) / 16.0;
    const double staged = (double)blocks * g.n_stages * (g.xbytes + g.wbytes) / cus / 64.0;   // 64 B/clk/CU
    return (double)rounds * (mfma + overhead) + staged;
}

const Variant* find_variant(const char* name, size_t len)
{
    for (int i = 0; i < kNumVariants; ++i)
        if (strlen(kVariants[i].name) == len && strncmp(kVariants[i].name, name, len) == 0) return &kVariants[i];
    return nullptr;
}

void fill_plan(const ConvArgs& a, const Variant& v, const IgemmGeom& g, LaunchPlan* out)
{
    static_assert(sizeof(IgemmGeom) <= sizeof(out->geom), "geometry does not fit the plan");
    out->id = KID_IGEMM;
    out->name = v.name;
    out->variant = (int)(&v - kVariants);
    out->grid_x = (unsigned)(g.row_blocks * g.img_blocks * g.k_blocks);
    out->grid_y = 1;
    out->block = (unsigned)((v.WM * v.WN + igemm_producer_waves(v.TM, v.TN, v.TAPS, v.UA, v.UB)) * 64);
    out->lds = lds_bytes(v, g);
    memcpy(out->geom, &g, sizeof g);
}

}  // namespace

#ifdef CVX_PHASE_TRACE
extern "C" int cvx_debug_set_phase_trace(unsigned long long* device_buffer)
{
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_phase_trace), &device_buffer, sizeof(device_buffer));
}
#endif

bool igemm_plan(const ConvArgs& a, const PlanEnv& env, LaunchPlan* out)
{
    if (a.dtype != DT_BF16 && a.dtype != DT_F16) return false;
    if (a.groups < 1 || a.C % a.groups || a.K % a.groups) return false;
    if (a.C / a.groups < 8) return false;                      // too few channels per group to fill an octet
    const long long xbytes = (long long)a.N * a.C * a.H * a.W * 2, ybytes = (long long)a.N * a.K * a.Ho * a.Wo * 2;
    if (xbytes >= (1LL << 31) || ybytes >= (1LL << 31)) return false;
    if (!env.aligned16) return false;
    const int HoWo = a.Ho * a.Wo;
    if (env.pin) {
        // "<variant>" or "<variant>,<NB>,<TH>"
        const char* comma = strchr(env.pin, ',');
        const Variant* v = find_variant(env.pin, comma ? (size_t)(comma - env.pin) : strlen(env.pin));
        if (!v) return false;
        const int PT = v->WM * v->TM * 32;
        int nb = 0, th = 0;
        if (comma) {
            if (sscanf(comma, ",%d,%d", &nb, &th) != 2) return false;
        } else if (HoWo <= PT) {
            nb = PT / HoWo < a.N ? PT / HoWo : a.N;
            th = a.Ho;
        } else {
            nb = 1;
            th = PT / a.Wo;
        }
        IgemmGeom g;
        if (!plan(a, *v, nb, th, &g)) return false;
        fill_plan(a, *v, g, out);
        return true;
    }
    double best = 1e300;
    const Variant* bv = nullptr;
    IgemmGeom bg;
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant& v = kVariants[i];
        const int PT = v.WM * v.TM * 32;
        if (a.Wo > PT) continue;
        const bool multi = HoWo <= PT;           // whole images fit: tile over images
        int hi = multi ? PT / HoWo : PT / a.Wo;
        if (multi) {
            // no more images per tile than the loader threads and the LDS can take (plan() checks both
            // exactly; this only keeps the search from walking through hundreds of hopeless sizes)
            const int OCT = v.CC / 8, PH = (a.Ho - 1) * a.stride_h + (a.R - 1) * a.dil_h + 1;
            const int WP = (a.W + 2 * a.pad_w + 7) & ~7;
            const long long upi = ((long long)PH * a.W + 7) / 8, slot_bytes = (long long)PH * WP * 18;
            const long long by_units = (long long)v.UA * 256 / (OCT * upi), by_lds = (LDS_LIMIT / 2) / (OCT * slot_bytes);
            if (by_units < hi) hi = (int)by_units;
            if (by_lds < hi) hi = (int)by_lds;
        }
        // only tile heights near the top matter: shorter tiles only add blocks
        for (int t = hi, tried = 0; t >= 1 && tried < 12; --t) {
            IgemmGeom g;
            if (!plan(a, v, multi ? t : 1, multi ? a.Ho : t, &g)) continue;
            ++tried;
            const double c = cost(a, v, g, env.cus);
            if (c < best) {
                best = c;
                bv = &v;
                bg = g;
            }
        }
    }
    if (!bv) return false;
    fill_plan(a, *bv, bg, out);
    return true;
}

hipError_t igemm_prepare()
{
    static const hipError_t status = [] {
        for (int i = 0; i < kNumVariants; ++i) {
            for (auto kern : {kVariants[i].kern_bf16, kVariants[i].kern_f16}) {
                hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_LIMIT);
                if (e != hipSuccess) return e;
            }
        }
        return hipSuccess;
    }();
    return status;
}

hipError_t igemm_launch(const ConvArgs& a, const LaunchPlan& p, hipStream_t s)
{
    hipError_t e = igemm_prepare();
    if (e != hipSuccess) return e;
    const Variant& v = kVariants[p.variant];
    IgemmGeom g;
    memcpy(&g, p.geom, sizeof g);
    auto kern = a.dtype == DT_BF16 ? v.kern_bf16 : v.kern_f16;
    hipLaunchKernelGGL(kern, dim3(p.grid_x), dim3(p.block), p.lds, s, a, g);
    return hipGetLastError();
}

}  // namespace cvx
