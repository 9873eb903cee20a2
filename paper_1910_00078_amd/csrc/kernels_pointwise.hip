// Pointwise (1x1 filter, unit stride, no padding) forward convolution on bf16 / fp16 MFMA for
// gfx950 (MI355X), with the bias / batch-norm / activation epilogue of Sec. V of the MIOpen paper
// applied to the accumulators before the single store.
//
// A 1x1 convolution is the GEMM  Y[n][k][pix] = sum_c Wt[k][c] * X[n][c][pix]  and, at the channel
// counts of residual networks, is bound by device-memory bandwidth, not by the matrix pipe.  The
// kernel is therefore organised around keeping the memory system busy without pause:
//
//   Persistent blocks   one block per compute unit; block b owns a contiguous span of the flattened
//                       (image, pixel) axis, so the blocks carry equal bytes, and walks it in pixel
//                       tiles.  The filters and epilogue constants are loaded into LDS once.
//   Direct-to-LDS loads two loader waves stream the input with global_load_lds (16 bytes per lane,
//                       no registers in between) into a ring of NS stage buffers, each CC channel
//                       rows x PT pixels in the tensor's own NCHW order.  The ring runs ahead of the
//                       multiply across tile boundaries; the loaders wait on their own load counter
//                       with an exact outstanding-load count, so NS-2 stages stay in flight.
//   Transposing reads   NCHW keeps pixels contiguous but the MFMA pixel operand wants 8 consecutive
//                       channels per lane.  ds_read_b64_tr_b16 does that exchange inside the LDS
//                       read (16 lanes x 4 pixels in, 4 channels x 1 pixel per lane out), so nothing
//                       is transposed in registers.  The 64-byte chunks of a stage row are XOR-
//                       swizzled with the row index so the four rows a read touches fall on
//                       different banks; the swizzle costs nothing, the loader just picks the global
//                       address that belongs at each LDS position.
//   Wave-private stores each multiply wave stages its 64-pixel x 64-filter results in its own LDS
//                       patch and writes them out itself as 128-byte rows; no block-wide barrier
//                       sits between the multiply and the store, and the loaders never wait for a
//                       store.
#include "cvx_device.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>

namespace cvx {

namespace pw {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) unsigned char lds_byte;

struct Geom {
    int HW;            // pixels per image
    int total_px;      // N * HW
    int span;          // pixels per block, a multiple of the tile width
    int stages_per_tile;   // C / CC
    int x_streaming;   // 1: input loads carry the nontemporal hint
    int w_off, ca_off, out_off, ring_off;   // LDS byte offsets
};

// Transposing LDS read.  Within each group of 16 lanes, lane s supplies the address of 4 consecutive
// 16-bit elements; with K = s / 4 and M = 4 * (s % 4) + {0..3} naming those elements, lane i of the
// group receives the four elements (K = 0..3, M = i).  The low three address bits are ignored.
__device__ __forceinline__ u32x2 lds_read_tr16(const unsigned char* p)
{
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(lds_byte*)p);
    return __builtin_bit_cast(u32x2, v);
}

// All of a wave's LDS reads have returned; then the block barrier.  Deliberately not a fence: the
// loader waves keep device loads in flight across it and the multiply waves keep stores in flight.
__device__ __forceinline__ void stage_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int N>
__device__ __forceinline__ void wait_loads_outstanding()
{
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

constexpr int ND = 2;             // loader waves
constexpr int OPITCH = 136;       // bytes per filter row of a wave's output patch: 64 pixels + 4 (bank spread)

// WM x WN multiply waves, each TM pixel sub-tiles (32 pixels) x TN filter sub-tiles (32 filters);
// CC channels per stage; NS ring slots.
template <int DT, int WM, int WN, int TM, int TN, int CC, int NS>
__global__ void __launch_bounds__((WM * WN + ND) * 64)
pointwise_kernel(ConvArgs a, Geom g)
{
    constexpr int NCW = WM * WN;
    constexpr int THREADS = (NCW + ND) * 64;
    constexpr int PT = WM * TM * 32;                 // pixels per tile
    constexpr int KT = WN * TN * 32;                 // filters per block
    constexpr int ROWB = PT * 2;                     // bytes per channel row of a stage
    constexpr int STAGE = CC * ROWB;
    constexpr int INSTR = STAGE / 1024;              // wave-wide 16-byte-per-lane loads per stage
    constexpr int U = INSTR / ND;                    // of which each loader wave issues this many
    constexpr int RPI = 1024 / ROWB;                 // channel rows one such load covers
    constexpr int KSTEPS = CC / 16;
    static_assert(PT >= 128 && PT <= 512 && (PT & (PT - 1)) == 0, "swizzle needs >= 4 chunks of 64 bytes per row");
    static_assert(INSTR % ND == 0 && (ND * RPI) % 4 == 0, "a lane keeps one swizzle phase");
    static_assert(TM % 2 == 0, "output patches hold two pixel sub-tiles");
    static_assert((NS - 2) * U <= 63, "outstanding loads must fit the counter");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    CVX_TRACE_MARK(0);
    warm_kernel_arguments<sizeof(ConvArgs) + sizeof(Geom)>();
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int HW = g.HW;
    const int k0 = blockIdx.y * KT;

    // this block's span of the flattened (image, pixel) axis
    const int Gb = blockIdx.x * g.span;
    if (Gb >= g.total_px) return;                                    // whole block, before any barrier
    const int Ge = min(Gb + g.span, g.total_px);
    const int n_tiles = (Ge - Gb + PT - 1) / PT;
    const int SPT = g.stages_per_tile;
    const int T = n_tiles * SPT;                                     // stages this block multiplies

    unsigned char* ws = smem + g.w_off;               // written by the multiply waves' prologue
    float* cas = (float*)(smem + g.ca_off);
    unsigned char* ring = smem + g.ring_off;

    if (wave >= NCW) {
        // =========================================================================================
        // loader waves
        // =========================================================================================
        const int dw = wave - NCW;
        const uint16_t* __restrict__ xg = (const uint16_t*)a.x;
        // LDS position of this lane inside a load: channel row (relative) and 16-byte unit of the row
        const int lane_row = (lane * 16) / ROWB;
        const int u16 = ((lane * 16) % ROWB) >> 4;
        const int rowlow = (dw * RPI + lane_row) & 3;               // row & 3, the same for every load of this wave
        const int px = (((u16 >> 2) ^ rowlow) << 5) + ((u16 & 3) << 3);   // pixel of the tile that belongs here
        const int Glast = Ge - 8;                                    // last whole 8-pixel chunk of the span

        int ld_tile = 0, ld_st = 0, ld_slot = 0;
        long long goff = 0;
        auto issue_stage = [&]() __attribute__((always_inline)) {
            if (ld_st == 0) {
                // pixels past the span re-read its last chunk: every lane always loads, so the
                // outstanding-load arithmetic below is exact, and the address stays inside x
                const int G = min(Gb + ld_tile * PT + px, Glast);
                const int n = G / HW;
                goff = (long long)n * a.C * HW + (G - n * HW);
            }
            const uint16_t* src = xg + goff + (long long)(ld_st * CC + dw * RPI + lane_row) * HW;
            lds_byte* dst = (lds_byte*)(ring + ld_slot * STAGE + dw * 1024);
            // The streaming hint keeps a large input from displacing the output lines waiting in L2; it
            // pays when the input is the larger tensor.
            if (g.x_streaming) {
#pragma unroll
                for (int u = 0; u < U; ++u)
                    __builtin_amdgcn_global_load_lds((const void*)(src + (long long)u * (ND * RPI) * HW),
                                                     (__attribute__((address_space(3))) void*)(dst + u * ND * 1024), 16, 0, 2);
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u)
                    __builtin_amdgcn_global_load_lds((const void*)(src + (long long)u * (ND * RPI) * HW),
                                                     (__attribute__((address_space(3))) void*)(dst + u * ND * 1024), 16, 0, 0);
            }
            if (++ld_st == SPT) { ld_st = 0; ++ld_tile; }
            if (++ld_slot == NS) ld_slot = 0;
        };

        const int ahead = min(NS - 1, T);
        for (int s = 0; s < ahead; ++s) issue_stage();
        CVX_TRACE_MARK_T(10, NCW * 64);
        if (ahead == NS - 1) wait_loads_outstanding<(NS - 2) * U>();
        else wait_loads_outstanding<0>();
        CVX_TRACE_MARK_T(11, NCW * 64);
        stage_barrier();                                             // filters, constants and stage 0 are in LDS
        for (int t = 0; t < T; ++t) {
            // slot (t-1) % NS was multiplied in the previous pass; refill it with stage t+NS-1, then
            // wait until stage t+1 has landed (at most NS-2 younger stages still in flight)
            if (t + NS - 1 < T) {
                issue_stage();
                wait_loads_outstanding<(NS - 2) * U>();
            } else {
                wait_loads_outstanding<0>();
            }
            stage_barrier();
        }
    } else {
        // =========================================================================================
        // multiply waves
        // =========================================================================================
        const int l32 = lane & 31, h = lane >> 5;
        const int gq = lane >> 4, s16 = lane & 15;
        const int wm = wave / WN, wn = wave % WN;
        const bool has_bn = a.bn_scale != nullptr;

        // pixel operand: byte offset inside a stage for sub-tile tm, k-step 0, first half
        int xa[TM];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int jt = wm * TM + tm;
            xa[tm] = (8 * h + (s16 >> 2)) * ROWB + ((jt ^ (s16 >> 2)) << 6) + ((gq & 1) << 5) + ((s16 & 3) << 3);
        }
        const unsigned char* wl = ws + ((size_t)h * KT + (wn * TN) * 32 + l32) * 16;
        unsigned char* ow = smem + g.out_off + wave * (TN * 32 * OPITCH);

        // ---- once per block (the loaders are already streaming the input): filters into LDS as
        //      [channel octet][filter] x 16 bytes, by direct-to-LDS loads whose per-lane device address
        //      does the reordering, and the epilogue constants.  Filter rows past K repeat row K-1:
        //      they only feed output columns that are never stored.
        {
            const uint16_t* __restrict__ wg = (const uint16_t*)a.w;
            constexpr int KCH = KT / 64;                             // 1 KiB chunks per channel octet
            const int chunks = (a.C >> 3) * KCH;
            for (int j = wave; j < chunks; j += NCW) {
                const int o = j / KCH, kl = (j - o * KCH) * 64 + lane;
                const uint16_t* src = wg + ((size_t)min(k0 + kl, a.K - 1) * a.C + o * 8);
                __builtin_amdgcn_global_load_lds((const void*)src, (__attribute__((address_space(3))) void*)(lds_byte*)(ws + j * 1024),
                                                 16, 0, 0);
            }
            for (int kl = tid; kl < KT; kl += NCW * 64) {
                const ChannelAffine c1 = channel_affine<DT>(a, min(k0 + kl, a.K - 1));
                cas[2 * kl] = c1.mul;
                cas[2 * kl + 1] = c1.add;
            }
            wait_loads_outstanding<0>();
        }
        CVX_TRACE_MARK(1);
        stage_barrier();                                             // filters, constants and stage 0 are in LDS
        CVX_TRACE_MARK(2);
        ChannelAffine ca[TN];
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            ca[tn].mul = cas[2 * ((wn * TN + tn) * 32 + l32)];
            ca[tn].add = cas[2 * ((wn * TN + tn) * 32 + l32) + 1];
        }
        f32x16 acc[TM][TN];
        auto seed = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const float sd = has_bn ? 0.0f : ca[tn].add;
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[tm][tn][r] = sd;
                }
        };
        seed();

        uint16_t* __restrict__ yg = (uint16_t*)a.y;
        // The wave's patch [TN*32 filters][64 pixels] -> device memory, 8 lanes (16 bytes each) per
        // filter row.  `tp` selects which pair of the wave's pixel sub-tiles the patch holds.
        auto flush_patch = [&](int tile, int tp) __attribute__((always_inline)) {
            const int G = Gb + tile * PT + (wm * TM + tp * 2) * 32 + (lane & 7) * 8;
            const bool live = G < Ge;
            const int n = G / HW;
            const size_t obase = ((size_t)n * a.K + k0 + wn * TN * 32) * HW + (G - n * HW);
            u32x4 v[TN * 4];
#pragma unroll
            for (int i = 0; i < TN * 4; ++i) {
                const unsigned char* p = ow + (i * 8 + (lane >> 3)) * OPITCH + (lane & 7) * 16;
                const u32x2 lo = *(const u32x2*)p, hi = *(const u32x2*)(p + 8);
                v[i] = u32x4{lo[0], lo[1], hi[0], hi[1]};
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < TN * 4; ++i) {
                const int row = i * 8 + (lane >> 3);
                // streaming store: the output is not read again by this kernel, and lines left dirty in
                // L2 would all have to be written back at the end of the kernel
                if (live && k0 + wn * TN * 32 + row < a.K) __builtin_nontemporal_store(v[i], (u32x4*)(yg + obase + (size_t)row * HW));
            }
        };
        auto finish_tile = [&](int tile, auto&& act_fn) __attribute__((always_inline)) {
#pragma unroll
            for (int tp = 0; tp < TM / 2; ++tp) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            float v[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const float t = acc[tp * 2 + t2][tn][4 * q4 + j];
                                v[j] = act_fn(has_bn ? fmaf(t, ca[tn].mul, ca[tn].add) : t);
                            }
                            *(u32x2*)(ow + (tn * 32 + l32) * OPITCH + (t2 * 32 + 8 * q4 + 4 * h) * 2) =
                                u32x2{pack2<DT>(v[0], v[1]), pack2<DT>(v[2], v[3])};
                        }
                flush_patch(tile, tp);
            }
        };

        // bias + ReLU / identity (the bias is already in the accumulators): round, then ReLU on the
        // packed pair, 1 instruction per value
        auto finish_tile_packed = [&](int tile, uint32_t floor2) __attribute__((always_inline)) {
#pragma unroll
            for (int tp = 0; tp < TM / 2; ++tp) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            const auto& t = acc[tp * 2 + t2][tn];
                            *(u32x2*)(ow + (tn * 32 + l32) * OPITCH + (t2 * 32 + 8 * q4 + 4 * h) * 2) =
                                u32x2{max_packed(pack2<DT>(t[4 * q4], t[4 * q4 + 1]), floor2),
                                      max_packed(pack2<DT>(t[4 * q4 + 2], t[4 * q4 + 3]), floor2)};
                        }
                flush_patch(tile, tp);
            }
        };

        int st = 0, tile = 0, slot = 0;
        for (int t = 0; t < T; ++t) {
            const unsigned char* xs = ring + slot * STAGE;
            const unsigned char* wst = wl + (size_t)st * (CC / 8) * KT * 16;
            u32x4 fa[KSTEPS][TM], fb[KSTEPS][TN];
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) fb[kk][tn] = *(const u32x4*)(wst + (kk * 2 * KT + tn * 32) * 16);
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    const u32x2 lo = lds_read_tr16(xs + xa[tm] + kk * 16 * ROWB);
                    const u32x2 hi = lds_read_tr16(xs + xa[tm] + kk * 16 * ROWB + 4 * ROWB);
                    fa[kk][tm] = u32x4{lo[0], lo[1], hi[0], hi[1]};
                }
            }
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) acc[tm][tn] = mfma_32x32x16<DT>(fa[kk][tm], fb[kk][tn], acc[tm][tn]);

            if (++st == SPT) {
                st = 0;
                if (!has_bn && (a.act == ACT_RELU || a.act == ACT_IDENTITY)) finish_tile_packed(tile, packed_floor(a.act == ACT_RELU));
                else if (a.act == ACT_RELU) finish_tile(tile, [](float v) { return fmaxf(v, 0.0f); });
                else if (a.act == ACT_IDENTITY) finish_tile(tile, [](float v) { return v; });
                else finish_tile(tile, [&](float v) { return activate(v, a.act, a.alpha); });
                seed();
                ++tile;
                if (tile <= 6) CVX_TRACE_MARK(2 + tile);
            }
            if (++slot == NS) slot = 0;
            stage_barrier();
        }
        CVX_TRACE_MARK(15);
    }
}

// ------------------------------------------------------------------------------------------------
constexpr int LDS_LIMIT = 160 * 1024;

struct Variant {
    const char* name;
    int WM, WN, TM, TN, CC, NS;
    void (*kern_bf16)(ConvArgs, Geom);
    void (*kern_f16)(ConvArgs, Geom);
};

#define PW_VARIANT(nm, WM, WN, TM, TN, CC, NS)                                                  \
    {nm, WM, WN, TM, TN, CC, NS, pointwise_kernel<DT_BF16, WM, WN, TM, TN, CC, NS>,               \
     pointwise_kernel<DT_F16, WM, WN, TM, TN, CC, NS>}

// name: pointwise_<pixels per tile>x<filters per block>_c<channels per stage>_r<ring slots>
const Variant kVariants[] = {
    PW_VARIANT("pointwise_256x64_c32_r5", 4, 1, 2, 2, 32, 5),
    PW_VARIANT("pointwise_256x64_c32_r3", 4, 1, 2, 2, 32, 3),
    PW_VARIANT("pointwise_128x128_c32_r6", 2, 2, 2, 2, 32, 6),
    PW_VARIANT("pointwise_128x256_c32_r6", 1, 4, 4, 2, 32, 6),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

struct Plan {
    const Variant* v;
    Geom g;
    int blocks, kblocks, lds;
};

bool plan_variant(const ConvArgs& a, const Variant& v, int cus, Plan* out)
{
    const int PT = v.WM * v.TM * 32, KT = v.WN * v.TN * 32, NCW = v.WM * v.WN;
    if (a.C % v.CC) return false;
    Geom g;
    g.HW = a.H * a.W;
    g.total_px = a.N * g.HW;
    g.stages_per_tile = a.C / v.CC;
    g.x_streaming = a.C > a.K ? 1 : 0;
    const long long wbytes = (long long)a.C * KT * 2;
    const long long stage = (long long)v.CC * PT * 2;
    long long off = 0;
    g.w_off = (int)off;            off += wbytes;
    g.ca_off = (int)off;           off += (long long)KT * 8;
    g.out_off = (int)off;          off += (long long)NCW * v.TN * 32 * OPITCH;
    off = (off + 1023) & ~1023LL;
    g.ring_off = (int)off;         off += stage * v.NS;
    if (off > LDS_LIMIT) return false;
    const int kblocks = (a.K + KT - 1) / KT;
    // Blocks get equal runs of whole tiles: a nearly empty last tile would still cost a block the
    // full latency of its stages, while leaving a few compute units idle costs nothing as long as
    // the rest keep device memory busy.
    const long long tiles = ((long long)g.total_px + PT - 1) / PT;
    const long long rounds = (tiles + cus - 1) / cus;
    const long long span = rounds * PT;
    const int blocks = (int)((g.total_px + span - 1) / span);
    g.span = (int)span;
    out->v = &v;
    out->g = g;
    out->blocks = blocks;
    out->kblocks = kblocks;
    out->lds = (int)off;
    return true;
}

bool choose(const ConvArgs& a, const PlanEnv& env, Plan* out)
{
    if (a.dtype != DT_BF16 && a.dtype != DT_F16) return false;
    if (a.groups != 1 || a.R != 1 || a.S != 1) return false;
    if (a.stride_h != 1 || a.stride_w != 1 || a.pad_h != 0 || a.pad_w != 0) return false;
    const long long HW = (long long)a.H * a.W;
    if (HW % 8 || HW > (1 << 24)) return false;                      // 16-byte pixel chunks never straddle images
    if ((long long)a.N * HW >= (1LL << 30)) return false;            // flattened pixel index stays in int
    if ((long long)a.N * HW * a.C >= (1LL << 31) || (long long)a.N * HW * a.K >= (1LL << 31)) return false;
    if (a.C % 32) return false;
    if (!env.aligned16) return false;
    bool found = false;
    Plan best;
    for (int i = 0; i < kNumVariants; ++i) {
        Plan p;
        if (!plan_variant(a, kVariants[i], env.cus, &p)) continue;
        if (env.pin) {                                               // developer pin: variant name
            if (strcmp(env.pin, kVariants[i].name) == 0) {
                *out = p;
                return true;
            }
            continue;
        }
        // least multiply work (filter columns, padding included), then fewest passes over the input,
        // then the most bytes in flight
        const auto key = [](const Plan& q) {
            const long long KT = q.v->WN * q.v->TN * 32, PT = q.v->WM * q.v->TM * 32;
            return ((long long)q.kblocks * KT * 64 + q.kblocks) * 1024 - (long long)q.v->NS * q.v->CC * PT * 2 / 1024;
        };
        if (!found || key(p) < key(best)) {
            best = p;
            found = true;
        }
    }
    if (found) *out = best;
    return found;
}

}  // namespace pw

#ifdef CVX_PHASE_TRACE
extern "C" int cvx_debug_set_phase_trace_pointwise(unsigned long long* device_buffer)
{
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_phase_trace), &device_buffer, sizeof(device_buffer));
}
#endif

bool pointwise_plan(const ConvArgs& a, const PlanEnv& env, LaunchPlan* out)
{
    static_assert(sizeof(pw::Geom) <= sizeof(out->geom), "geometry does not fit the plan");
    pw::Plan p;
    if (!pw::choose(a, env, &p)) return false;
    out->id = KID_POINTWISE;
    out->name = p.v->name;
    out->variant = (int)(p.v - pw::kVariants);
    out->grid_x = (unsigned)p.blocks;
    out->grid_y = (unsigned)p.kblocks;
    out->block = (unsigned)((p.v->WM * p.v->WN + pw::ND) * 64);
    out->lds = p.lds;
    memcpy(out->geom, &p.g, sizeof p.g);
    return true;
}

hipError_t pointwise_prepare()
{
    static const hipError_t status = [] {
        for (int i = 0; i < pw::kNumVariants; ++i) {
            for (auto kern : {pw::kVariants[i].kern_bf16, pw::kVariants[i].kern_f16}) {
                hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, pw::LDS_LIMIT);
                if (e != hipSuccess) return e;
            }
        }
        return hipSuccess;
    }();
    return status;
}

hipError_t pointwise_launch(const ConvArgs& a, const LaunchPlan& p, hipStream_t s)
{
    hipError_t e = pointwise_prepare();
    if (e != hipSuccess) return e;
    const pw::Variant& v = pw::kVariants[p.variant];
    pw::Geom g;
    memcpy(&g, p.geom, sizeof g);
    auto kern = a.dtype == DT_BF16 ? v.kern_bf16 : v.kern_f16;
    hipLaunchKernelGGL(kern, dim3(p.grid_x, p.grid_y), dim3(p.block), p.lds, s, a, g);
    return hipGetLastError();
}

}  // namespace cvx
