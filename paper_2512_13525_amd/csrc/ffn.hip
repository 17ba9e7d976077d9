// a5: grouped expert FFN over the activated experts only (Janus Sec. 2.2: an expert is a
// fused gate/up GEMM and a down GEMM; at decode sizes the layer is bound by streaming the
// activated experts' weights from HBM, so latency follows the activated-expert count).
//
// bf16 path: ONE persistent kernel for both GEMM stages.
//
// Weights are consumed in a tile-packed layout: a 16-row x 32-column tile of a weight matrix
// is stored as the 1 KiB image of the MFMA A-operand of one wavefront (lane l holds row l%16,
// columns (l/16)*8 .. +7), and the two 16-row tiles a work unit multiplies together
// (16 gate + 16 up channels in stage 1, 32 output channels in stage 2) alternate per K-step,
// so a unit is one contiguous run of 2 KiB steps read with fully coalesced 128-bit loads
// straight into MFMA registers.  Tokens are the B operand (lane l holds token l%16, the same
// 8 columns), fetched from L2 (X through `perm`, or the intermediate `act`) and shared by
// both MFMAs of the step.  The 16x16 fp32 result leaves lane l with 4 consecutive output
// channels (l/16)*4.. of token l%16.
//
// Work decomposition.  Nothing about the activated set is known on the host, so every
// workgroup first compacts the activated slots from slot_off.  The work of a stage is the
// flat sequence  slot -> unit -> pass (32 tokens) -> quad (4 K-steps, one per wavefront);
// it is cut into gridDim equal ranges of quads, one per persistent workgroup, whatever the
// number of activated experts (a perfectly balanced split: the layer's latency then follows
// the activated-expert count down to a single expert).  A workgroup's 4 wavefronts take the
// 4 K-steps of a quad (split-K), keep a ring of kRing steps of loads in flight and meet in
// LDS at the end of a unit.  A unit cut by a range boundary is finished by the workgroup that
// holds its first quad (the last segment of that workgroup's range): every other part is the
// first segment of a later workgroup's range, stores its fp32 partial tile in a private
// workspace slot and bumps the unit's arrival counter; the finisher polls the counter (the
// parts are ready long before), adds the parts in workgroup order (so the sum is deterministic)
// and runs the epilogue.  Counter bumps are sent one segment late, when the stores they
// announce are known to be acknowledged, so no wavefront stalls on a store round trip.
// SiLU(gate)*up is rounded to bf16 once and written to `act`.
//
// Stage 2 of a slot may start only when all stage-1 units of that slot are done: a per-slot
// counter in the workspace header is bumped by every finished stage-1 unit and polled by
// stage 2.  `act`, the partial tiles and the counters are written and read with agent-scope
// (L2-coherent) accesses because the 8 XCDs do not share an L2, so no cache write-back or
// invalidation is ever issued; a writer waits for its stores to be acknowledged before it
// bumps a counter.  Every workgroup finishes all of its stage-1 work before it polls, and
// the grid is never larger than what is resident at once, so every awaited unit belongs to
// a running workgroup that never waits itself.  The poll is bounded all the same: on overrun
// the workgroup raises the error word of the header and carries on, so that every wave
// reaches the end of the kernel.  The last stage-2 unit of a slot clears that slot's
// counters, and the finisher of a cut unit clears its arrival counter, for the next call.
//
// Slots without requests are never compacted into the work list: their weights are not read.
//
// fp32 path (correctness configuration): plain wave-per-output-row dot products, two kernels.
#include <stdlib.h>

#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kTokTiles = 2;            // token tiles (of 16) per pass
constexpr int kPassTok = kTokTiles * 16;

constexpr int kRing = 2;                // K-steps of loads each wavefront keeps in flight
constexpr int kFfnThreads = 256;
constexpr int kMaxGrid = 1024;          // upper bound of the persistent grid
constexpr int kTokCacheSlots = 64;      // activated slots whose first-pass token rows are cached in LDS

// Workspace layout (bytes):
//   [0, kCtrlBytes)            header: int [1] = error word; slot s owns the 128-byte line at int
//                              offset kCtrlSlot0 + s*kCtrlStride ([0] stage-1 units done, [1] stage-2
//                              units done); arrival counters of cut units at int offset kCtrlArrive0
//                              + stage*kMaxGrid + (first workgroup of the unit)
//   [kCtrlBytes, +kPartBytes)  partial tiles [stage][workgroup][2][kTokTiles][2][64] x 16 B
//   [kCtrlBytes + kPartBytes, ...)  act
constexpr int kCtrlStride = 32;
constexpr int kCtrlSlot0 = 64;
constexpr int kCtrlArrive0 = kCtrlSlot0 + MOE_MAX_SLOTS * kCtrlStride;
constexpr int kCtrlInts = kCtrlArrive0 + 2 * kMaxGrid;
constexpr size_t kCtrlBytes = (static_cast<size_t>(kCtrlInts) * 4 + 255) / 256 * 256;
constexpr size_t kPartPerWg = 2 * 4 * kTokTiles * 2 * 64;              // f32x4 elements: 2 parts x (4 units x kTokTiles) x 2 halves
constexpr size_t kPartBytes = 2 * static_cast<size_t>(kMaxGrid) * kPartPerWg * 16;

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// ------------------------------------------------------------------ packing
// W13 [C, 2*d_e, d_h] -> [C][d_e/16][d_h/32][2 (gate, up)][64 lanes][8]
__global__ void pack_w13_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                int C, int d_h, int d_e) {
    const int JT = d_e / 16, KS = d_h / 32;
    const size_t n = static_cast<size_t>(C) * JT * KS * 2 * 64;
    for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < n;
         i += static_cast<size_t>(gridDim.x) * blockDim.x) {
        const int lane = i % 64;
        size_t r = i / 64;
        const int gu = r % 2; r /= 2;
        const int kk = r % KS; r /= KS;
        const int jt = r % JT;
        const int s = r / JT;
        const size_t row = static_cast<size_t>(s) * 2 * d_e + static_cast<size_t>(gu) * d_e + jt * 16 + (lane & 15);
        const size_t col = static_cast<size_t>(kk) * 32 + (lane >> 4) * 8;
        dst[i] = src[(row * d_h + col) / 8];
    }
}

// W2 [C, d_h, d_e] -> [C][d_h/32][d_e/32][2 (rows 0-15, rows 16-31)][64 lanes][8]
__global__ void pack_w2_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                               int C, int d_h, int d_e) {
    const int IT = d_h / 32, KS = d_e / 32;
    const size_t n = static_cast<size_t>(C) * IT * KS * 2 * 64;
    for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < n;
         i += static_cast<size_t>(gridDim.x) * blockDim.x) {
        const int lane = i % 64;
        size_t r = i / 64;
        const int half = r % 2; r /= 2;
        const int kk = r % KS; r /= KS;
        const int it = r % IT;
        const int s = r / IT;
        const size_t row = static_cast<size_t>(s) * d_h + it * 32 + half * 16 + (lane & 15);
        const size_t col = static_cast<size_t>(kk) * 32 + (lane >> 4) * 8;
        dst[i] = src[(row * d_e + col) / 8];
    }
}

__global__ void fill_zero_kernel(int *p, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0;
}

// ------------------------------------------------------------------ fused bf16 kernel
struct FfnArgs {
    const uint16_t *X;
    const bf16x8 *W13p;
    const bf16x8 *W2p;
    const int32_t *slot_off;
    const int32_t *perm;
    int *ctrl;
    f32x4 *part;
    uint16_t *act;
    float *Yp;
    int k, C, d_h, d_e;
    int act_stride;                      // elements between rows of act: a multiple of 64 (128-byte lines)
    int spin_limit;
};

// agent-scope (L2-coherent across XCDs) 16-byte accesses.  The compiler offers agent-scope
// atomics up to 64 bits only; the 128-bit forms are the same instructions with the sc1 bit, so
// that a wavefront moves a whole 1 KiB tile with one fully coalesced request.  The caller
// waits (s_waitcnt vmcnt(0)) before it relies on a store having landed; the load waits itself.
__device__ __forceinline__ void store_coherent(f32x4 *p, f32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}

__device__ __forceinline__ f32x4 load_coherent(const f32x4 *p) {
    f32x4 v;
    asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
    return v;
}

// Workgroup barrier for LDS exchange only: waits for this wavefront's LDS traffic, not for its
// global loads (the prefetched weights of the next segment stay in flight across it).
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + __expf(-g)) * u; }


struct FfnShared {
    f32x4 *red;                              // [wave][unit of the group][token tile][lane], one half at a time
    int slot[MOE_MAX_SLOTS];                 // activated slots, ascending
    int lo[MOE_MAX_SLOTS];                   // first request row of the slot
    int m[MOE_MAX_SLOTS];                    // requests of the slot
    int pre[MOE_MAX_SLOTS + 1];              // passes before activated slot j
    int tok[kTokCacheSlots][kPassTok];       // token row of the first-pass requests
    int a_g;
    int flag;
#ifdef MOE_FFN_TRACE
    long long wait_ticks;
    int tr_n;
#endif
};

// One segment = quads [qa, qb) of one group of R units for one pass of token tiles.  A K-step
// of the group is R x 2 weight fragments (R x 2 KiB) against the same token fragment(s).
// STAGE1: gate/up units (16 intermediate channels each); otherwise down units (32 output
// channels each).
#ifdef MOE_FFN_TRACE
// debug build only: thread 0 of every workgroup logs (tag, time) pairs into the unused second
// partial slot of its workgroup
#define MOE_TR(tag)                                                                              \
    if (threadIdx.x == 0) {                                                                      \
        long long *tr_ = reinterpret_cast<long long *>(a.part + blockIdx.x * kPartPerWg + kPartPerWg / 2); \
        const int n_ = sh.tr_n;                                                                  \
        if (n_ < 250) { tr_[2 + 2 * n_] = (tag); tr_[3 + 2 * n_] = wall_clock64(); sh.tr_n = n_ + 1; tr_[0] = n_ + 1; } \
    }
#else
#define MOE_TR(tag)
#endif

struct SegDesc {
    int j, pass, g_idx, qa, qb;
    int u0;                                  // first quad of the group in the stage's flat order
};

// Signals a workgroup owes for stores it has issued but not yet seen acknowledged.  They are sent
// one segment later, after the next streaming loop has drained (s_waitcnt vmcnt(0) is free there),
// so that no wavefront ever stalls on a store round trip.
struct Pending {
    int *arrive;       // arrival counter of a cut group this workgroup contributed a part to
    int *slot_done;    // stage-1 counter of a slot ...
    int slot_units;    // ... and the units finished for it
};

__device__ __forceinline__ void flush_pending(Pending &pd) {
    if (pd.arrive) __hip_atomic_fetch_add(pd.arrive, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (pd.slot_done) __hip_atomic_fetch_add(pd.slot_done, pd.slot_units, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    pd.arrive = nullptr;
    pd.slot_done = nullptr;
    pd.slot_units = 0;
}

// This wave's K-steps of a segment: kk = 4*(qa+i) + wave, i in [0, n_i)
__device__ __forceinline__ int seg_steps(const SegDesc &d, int KS, int QU, int wave) {
    int n_i = d.qb - d.qa;
    if (d.qb == QU && 4 * (QU - 1) + wave >= KS) n_i -= 1;
    return n_i;
}

template <bool STAGE1, int R>
__device__ __forceinline__ const bf16x8 *seg_weights(const FfnArgs &a, const FfnShared &sh, const SegDesc &d,
                                                     int wave, int lane) {
    const int n_s = STAGE1 ? a.d_e / 16 : a.d_h / 32;
    const int KS = (STAGE1 ? a.d_h : a.d_e) / 32;
    return (STAGE1 ? a.W13p : a.W2p) +
           ((static_cast<size_t>(sh.slot[d.j]) * n_s + static_cast<size_t>(d.g_idx) * R) * KS + 4 * d.qa + wave) * 128 + lane;
}

// First kRing K-steps of a segment's weights into the ring (issued as early as possible: before
// the previous segment's reduction and epilogue, so that their latency hides behind them).
template <int R>
__device__ __forceinline__ void seg_prefetch(const bf16x8 *wp, size_t unit_stride, int n_i, bf16x8 (*wr)[R][2]) {
#pragma unroll
    for (int d = 0; d < kRing; ++d) {
        if (d < n_i) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                wr[d][r][0] = wp[r * unit_stride + static_cast<size_t>(d) * 512];
                wr[d][r][1] = wp[r * unit_stride + static_cast<size_t>(d) * 512 + 64];
            }
        }
    }
}

template <bool STAGE1, int R>
__device__ __forceinline__ void ffn_segment(const FfnArgs &a, FfnShared &sh, const SegDesc &cur, const SegDesc &nxt,
                                            bool has_next, bf16x8 (*wr)[R][2], Pending &pd, int Q, int G,
                                            int wave, int lane) {
    const int j = cur.j, pass = cur.pass, g_idx = cur.g_idx, qa = cur.qa, qb = cur.qb;
    const int u0 = cur.u0;
    const int n = lane & 15, q4 = lane >> 4;
    const int n1 = a.d_e / 16, n2 = a.d_h / 32;
    const int KS = (STAGE1 ? a.d_h : a.d_e) / 32;
    const int QU = (KS + 3) >> 2;
    const int s = sh.slot[j], lo = sh.lo[j], m = sh.m[j];
    const int tile0 = pass * kTokTiles;
    const int n_tiles = (m + 15) >> 4;
    const int nt = min(kTokTiles, n_tiles - tile0);
    int *slot_ctrl = a.ctrl + kCtrlSlot0 + s * kCtrlStride;
    const size_t unit_stride = static_cast<size_t>(KS) * 128;      // 16-byte chunks between consecutive units
    const int n_i = seg_steps(cur, KS, QU, wave);
    const bf16x8 *wp = seg_weights<STAGE1, R>(a, sh, cur, wave, lane);   // its first kRing steps are already in flight
    MOE_TR((STAGE1 ? 100 : 200) + 0)

    if (!STAGE1) {
        // every stage-1 unit of this slot must have published its part of `act`
        if (threadIdx.x == 0) {
#ifdef MOE_FFN_TRACE
            const long long w0 = wall_clock64();
#endif
            const int need = n1 * (sh.pre[j + 1] - sh.pre[j]);
            int spins = 0;
            while (__hip_atomic_load(&slot_ctrl[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < need) {
                __builtin_amdgcn_s_sleep(16);
                if (++spins > a.spin_limit) {
                    __hip_atomic_store(&a.ctrl[1], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
            }
#ifdef MOE_FFN_TRACE
            sh.wait_ticks += wall_clock64() - w0;
#endif
        }
        lds_barrier();
    }

    // ---- token rows of this pass (B operand)
    const uint16_t *bp[kTokTiles];
#pragma unroll
    for (int t = 0; t < kTokTiles; ++t) {
        const int idx = (tile0 + t) * 16 + n;
        const int r = idx < m ? idx : tile0 * 16;                    // padding lanes reuse a valid row
        if (STAGE1) {
            int tok;
            if (pass == 0 && j < kTokCacheSlots) tok = sh.tok[j][r];
            else tok = a.perm[lo + r] / a.k;
            bp[t] = a.X + static_cast<size_t>(tok) * a.d_h + (4 * qa + wave) * 32 + q4 * 8;
        } else {
            bp[t] = a.act + static_cast<size_t>(lo + r) * a.act_stride + (4 * qa + wave) * 32 + q4 * 8;
        }
    }
    bf16x8 br[kRing][kTokTiles];
#pragma unroll
    for (int d = 0; d < kRing; ++d) {
        if (d < n_i) {
#pragma unroll
            for (int t = 0; t < kTokTiles; ++t)
                if (t < nt) br[d][t] = *reinterpret_cast<const bf16x8 *>(bp[t] + d * 128);
        }
    }

    MOE_TR((STAGE1 ? 100 : 200) + 1)
    f32x4 acc[R][kTokTiles][2];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int t = 0; t < kTokTiles; ++t) { acc[r][t][0] = f32x4{0, 0, 0, 0}; acc[r][t][1] = f32x4{0, 0, 0, 0}; }

#define MOE_STEP(d, i, REFILL)                                                        \
    {                                                                                 \
        /* consume ring entry d, then refill the same registers (no copies) */         \
        _Pragma("unroll") for (int r = 0; r < R; ++r) {                               \
            _Pragma("unroll") for (int t = 0; t < kTokTiles; ++t) {                   \
                if (t < NT_) {                                                        \
                    acc[r][t][0] = mfma16(wr[d][r][0], br[d][t], acc[r][t][0]);       \
                    acc[r][t][1] = mfma16(wr[d][r][1], br[d][t], acc[r][t][1]);       \
                }                                                                     \
            }                                                                         \
        }                                                                             \
        if (REFILL) {                                                                 \
            const size_t o_ = static_cast<size_t>((i) + kRing);                       \
            _Pragma("unroll") for (int r = 0; r < R; ++r) {                           \
                wr[d][r][0] = wp[r * unit_stride + o_ * 512];                         \
                wr[d][r][1] = wp[r * unit_stride + o_ * 512 + 64];                    \
            }                                                                         \
            _Pragma("unroll") for (int t = 0; t < kTokTiles; ++t)                     \
                if (t < NT_) br[d][t] = *reinterpret_cast<const bf16x8 *>(bp[t] + o_ * 128); \
        }                                                                             \
    }
#define MOE_STREAM(NTV)                                                               \
    {                                                                                 \
        constexpr int NT_ = NTV;                                                      \
        int i0 = 0;                                                                   \
        for (; i0 + 2 * kRing <= n_i; i0 += kRing) {                                  \
            _Pragma("unroll") for (int d = 0; d < kRing; ++d) MOE_STEP(d, i0 + d, true) \
        }                                                                             \
        for (; i0 < n_i; i0 += kRing) {                                               \
            _Pragma("unroll") for (int d = 0; d < kRing; ++d) {                       \
                const int i = i0 + d;                                                 \
                if (i < n_i) MOE_STEP(d, i, i + kRing < n_i)                          \
            }                                                                         \
        }                                                                             \
    }
    if (nt == 1) MOE_STREAM(1) else MOE_STREAM(2)
#undef MOE_STREAM
#undef MOE_STEP

    // every load of this segment has been consumed, so this costs nothing; it also means that the
    // stores of the previous segment (partial tiles, `act`) have been acknowledged
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    MOE_TR((STAGE1 ? 100 : 200) + 2)

    // ---- the next segment's first weights go out before this one's reduction and epilogue
    if (has_next)
        seg_prefetch<R>(seg_weights<STAGE1, R>(a, sh, nxt, wave, lane), unit_stride, seg_steps(nxt, KS, QU, wave), wr);

    // ---- the 4 wavefronts' partial tiles meet in LDS, one half (gate | up, rows 0-15 | 16-31) at a
    // time; wave w then owns the (unit, token tile) pairs w and w+4
    f32x4 res[2][2];                                                 // [pair slot][half]
    if (R == 1) {
        // both halves at once: red is [wave][half][token tile][lane]
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int t = 0; t < kTokTiles; ++t)
                if (t < nt) sh.red[((wave * 2 + h) * kTokTiles + t) * 64 + lane] = acc[0][t][h];
        lds_barrier();
        // past this barrier every wavefront has seen its earlier stores acknowledged
        if (threadIdx.x == 0) flush_pending(pd);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            f32x4 v = f32x4{0, 0, 0, 0};
            if (wave < nt) {
                v = sh.red[(h * kTokTiles + wave) * 64 + lane];
#pragma unroll
                for (int w = 1; w < 4; ++w) v += sh.red[((w * 2 + h) * kTokTiles + wave) * 64 + lane];
            }
            res[0][h] = v;
            res[1][h] = f32x4{0, 0, 0, 0};
        }
        lds_barrier();
    } else {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int t = 0; t < kTokTiles; ++t)
                    if (t < nt) sh.red[((wave * R + r) * kTokTiles + t) * 64 + lane] = acc[r][t][h];
            lds_barrier();
            if (h == 0 && threadIdx.x == 0) flush_pending(pd);
#pragma unroll
            for (int ps = 0; ps < 2; ++ps) {
                const int p = wave + 4 * ps;
                const int r = p / kTokTiles, t = p % kTokTiles;
                f32x4 v = f32x4{0, 0, 0, 0};
                if (p < R * kTokTiles && t < nt) {
                    v = sh.red[(r * kTokTiles + t) * 64 + lane];
#pragma unroll
                    for (int w = 1; w < 4; ++w) v += sh.red[((w * R + r) * kTokTiles + t) * 64 + lane];
                }
                res[ps][h] = v;
            }
            lds_barrier();
        }
    }

    MOE_TR((STAGE1 ? 100 : 200) + 3)
    const bool whole = qa == 0 && qb == QU;
    bool finish = whole;
    if (!whole) {
        // A group cut by a range boundary.  The part that holds the group's first quad finishes it:
        // that part is the last segment of its workgroup's range, while every other part is the
        // first segment of a later workgroup's range, so the others are ready long before.
        const int b_first = static_cast<int>(((u0 + 1LL) * G - 1) / Q);
        const int b_last = static_cast<int>((static_cast<long long>(u0 + QU) * G - 1) / Q);
        int *arrive = a.ctrl + kCtrlArrive0 + (STAGE1 ? 0 : kMaxGrid) + b_first;
        const size_t part0 = STAGE1 ? 0 : static_cast<size_t>(kMaxGrid);
        if (qa != 0) {
            f32x4 *mine = a.part + (part0 + blockIdx.x) * kPartPerWg;
#pragma unroll
            for (int ps = 0; ps < 2; ++ps) {
                const int p = wave + 4 * ps;
                if (p < R * kTokTiles && p % kTokTiles < nt) {
                    store_coherent(mine + (p * 2 + 0) * 64 + lane, res[ps][0]);
                    store_coherent(mine + (p * 2 + 1) * 64 + lane, res[ps][1]);
                }
            }
            if (threadIdx.x == 0) pd.arrive = arrive;                // sent once the stores are acknowledged
        } else {
            if (threadIdx.x == 0) {
                int spins = 0;
                while (__hip_atomic_load(arrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < b_last - b_first) {
                    __builtin_amdgcn_s_sleep(8);
                    if (++spins > a.spin_limit) {
                        __hip_atomic_store(&a.ctrl[1], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                }
                __hip_atomic_store(arrive, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next call
            }
            lds_barrier();
            finish = true;
#pragma unroll
            for (int ps = 0; ps < 2; ++ps) {
                const int p = wave + 4 * ps;
                if (p < R * kTokTiles && p % kTokTiles < nt) {
                    f32x4 v0 = res[ps][0], v1 = res[ps][1];
                    for (int b = b_first + 1; b <= b_last; ++b) {    // fixed order: deterministic sum
                        const f32x4 *q = a.part + (part0 + b) * kPartPerWg;
                        v0 += load_coherent(q + (p * 2 + 0) * 64 + lane);
                        v1 += load_coherent(q + (p * 2 + 1) * 64 + lane);
                    }
                    res[ps][0] = v0; res[ps][1] = v1;
                }
            }
        }
    }

    if (finish) {
#pragma unroll
        for (int ps = 0; ps < 2; ++ps) {
            const int p = wave + 4 * ps;
            const int r = p / kTokTiles, t = p % kTokTiles;
            const int idx = (tile0 + t) * 16 + n;
            if (p < R * kTokTiles && t < nt && idx < m) {
                const int t_idx = g_idx * R + r;
                const f32x4 r0 = res[ps][0], r1 = res[ps][1];
                if (STAGE1) {
                    // agent-scope store: visible to the other XCDs once acknowledged
                    const uint64_t o =
                        static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(r0[0], r1[0]))) |
                        static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(r0[1], r1[1]))) << 16 |
                        static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(r0[2], r1[2]))) << 32 |
                        static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(r0[3], r1[3]))) << 48;
                    __hip_atomic_store(reinterpret_cast<uint64_t *>(a.act + static_cast<size_t>(lo + idx) * a.act_stride +
                                                                    t_idx * 16 + q4 * 4),
                                       o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    float *y = a.Yp + static_cast<size_t>(lo + idx) * a.d_h + t_idx * 32 + q4 * 4;
                    *reinterpret_cast<f32x4 *>(y) = r0;
                    *reinterpret_cast<f32x4 *>(y + 16) = r1;
                }
            }
        }
        MOE_TR((STAGE1 ? 100 : 200) + (whole ? 4 : 5))
        if (threadIdx.x == 0) {
            if (STAGE1) {
                // the slot's counter is bumped once these `act` stores are acknowledged
                pd.slot_done = &slot_ctrl[0];
                pd.slot_units = R;
            } else {
                const int total2 = n2 * (sh.pre[j + 1] - sh.pre[j]);
                if (__hip_atomic_fetch_add(&slot_ctrl[1], R, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == total2 - R) {
                    // last stage-2 group of the slot: every other group of the slot has passed its wait
                    __hip_atomic_store(&slot_ctrl[0], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(&slot_ctrl[1], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
}

template <bool STAGE1, int R>
__device__ __forceinline__ void ffn_stage(const FfnArgs &a, FfnShared &sh, int wave, int lane) {
    const int a_g = sh.a_g;
    const int n_g = (STAGE1 ? a.d_e / 16 : a.d_h / 32) / R;          // groups of R units per slot
    const int KS = (STAGE1 ? a.d_h : a.d_e) / 32;
    const int QU = (KS + 3) >> 2;
    const int per_pass = n_g * QU;                                   // quads of one pass of one slot
    const int Q = sh.pre[a_g] * per_pass;                            // quads of the stage (the host bounds it below 2^31)
    if (Q == 0) return;
    // at most one workgroup per quad, so that no range is empty and every workgroup that a
    // cut group counts on does arrive
    const int G = min(static_cast<int>(gridDim.x), Q);
    if (static_cast<int>(blockIdx.x) >= G) return;
    int q = static_cast<int>(static_cast<long long>(blockIdx.x) * Q / G);
    const int q_hi = static_cast<int>((blockIdx.x + 1LL) * Q / G);
    int j = 0;
    auto describe = [&](int at) {
        while (sh.pre[j + 1] * per_pass <= at) ++j;
        // inside a slot: group -> pass -> quad, so that the passes of a group (more than 32 tokens
        // on one expert) re-read its weights back to back, from L2 rather than from HBM
        const int rel = at - sh.pre[j] * per_pass;
        const int per_group = (sh.pre[j + 1] - sh.pre[j]) * QU;
        SegDesc d;
        d.j = j;
        d.g_idx = rel / per_group;
        const int rel2 = rel - d.g_idx * per_group;
        d.pass = rel2 / QU;
        d.qa = rel2 - d.pass * QU;
        d.qb = min(QU, d.qa + (q_hi - at));
        d.u0 = at - d.qa;
        return d;
    };
    bf16x8 wr[kRing][R][2];
    Pending pd{nullptr, nullptr, 0};                                 // meaningful in thread 0 only
    SegDesc cur = describe(q);
    seg_prefetch<R>(seg_weights<STAGE1, R>(a, sh, cur, wave, lane), static_cast<size_t>(KS) * 128,
                    seg_steps(cur, KS, QU, wave), wr);
    while (true) {
        q += cur.qb - cur.qa;
        const bool has_next = q < q_hi;
        SegDesc nxt = cur;
        if (has_next) nxt = describe(q);
        ffn_segment<STAGE1, R>(a, sh, cur, nxt, has_next, wr, pd, Q, G, wave, lane);
        if (!has_next) break;
        cur = nxt;
    }
    // the last segment's signals
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) flush_pending(pd);
}

// Activated slots in slot order, their request rows, the prefix of passes (PT tokens per pass)
// and the token rows of each slot's first requests.
template <int PT>
__device__ __forceinline__ void ffn_prologue(const FfnArgs &a, FfnShared &sh, int wave, int lane) {
    // ---- activated slots in slot order, their request rows, and the pass prefix
    if (wave == 0) {
        int base = 0, passes = 0;
        for (int s0 = 0; s0 < a.C; s0 += MOE_WAVE) {
            const int s = s0 + lane;
            const int lo = s < a.C ? a.slot_off[s] : 0;
            const int m = s < a.C ? a.slot_off[s + 1] - lo : 0;
            const bool on = m > 0;
            const uint64_t mask = __ballot(on);
            const int p = on ? (m + PT - 1) / PT : 0;
            int incl = p;                                            // inclusive scan of passes over lanes
#pragma unroll
            for (int d = 1; d < MOE_WAVE; d <<= 1) {
                const int o = __shfl_up(incl, d, MOE_WAVE);
                if (lane >= d) incl += o;
            }
            if (on) {
                const int jj = base + __popcll(mask & moe::lanemask_lt());
                sh.slot[jj] = s; sh.lo[jj] = lo; sh.m[jj] = m;
                sh.pre[jj] = passes + incl - p;
            }
            base += __popcll(mask);
            passes += __shfl(incl, MOE_WAVE - 1, MOE_WAVE);
        }
        if (lane == 0) { sh.a_g = base; sh.pre[base] = passes; }
    }
    __syncthreads();
    {
        const int n_cache = min(sh.a_g, kTokCacheSlots) * kPassTok;
        for (int i = threadIdx.x; i < n_cache; i += kFfnThreads) {
            const int j = i / kPassTok, r = i - j * kPassTok;
            sh.tok[j][r] = a.perm[sh.lo[j] + (r < sh.m[j] ? r : 0)] / a.k;
        }
    }
    __syncthreads();

}

constexpr int kFfnWgPerCu = 2;          // resident workgroups per CU the register budget is sized for
constexpr int RMAX = 4;                 // largest group of units multiplied against the same token fragments

__global__ __launch_bounds__(kFfnThreads, kFfnWgPerCu)
void ffn_fused_kernel(FfnArgs a) {
    __shared__ FfnShared sh;
    __shared__ f32x4 red_lds[4 * (RMAX > 2 ? RMAX : 2) * kTokTiles * 64];
    if (threadIdx.x == 0) sh.red = red_lds;
#ifdef MOE_FFN_TRACE
    const long long t0 = wall_clock64();
    if (threadIdx.x == 0) { sh.wait_ticks = 0; sh.tr_n = 0; }
#endif
    // `act` is read with ordinary loads, and only after it is complete: nothing stale can be cached,
    // because caches are invalidated at the kernel boundary and no line of `act` is read early
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: scalar control flow
    const int lane = threadIdx.x & 63;

    ffn_prologue<kPassTok>(a, sh, wave, lane);

    // Units are multiplied in groups of R = 4, 2 or 1 against the same token fragments: larger
    // groups re-read the tokens less often, but a group is the unit of the cross-workgroup fix-up,
    // so R is kept small enough that a workgroup's range spans at least ~2 groups.
    const int n1 = a.d_e / 16, n2 = a.d_h / 32;
    const long long passes = sh.pre[sh.a_g];
    const long long grid = gridDim.x;
#ifdef MOE_FFN_TRACE
    const long long t1 = wall_clock64();
#endif
    if (RMAX >= 4 && n1 % 4 == 0 && passes * n1 >= 8 * grid) ffn_stage<true, (RMAX >= 4 ? 4 : 1)>(a, sh, wave, lane);
    else if (RMAX >= 2 && n1 % 2 == 0 && passes * n1 >= 4 * grid) ffn_stage<true, (RMAX >= 2 ? 2 : 1)>(a, sh, wave, lane);
    else ffn_stage<true, 1>(a, sh, wave, lane);
#ifdef MOE_FFN_TRACE
    const long long t2 = wall_clock64();
#endif
    if (RMAX >= 4 && n2 % 4 == 0 && passes * n2 >= 8 * grid) ffn_stage<false, (RMAX >= 4 ? 4 : 1)>(a, sh, wave, lane);
    else if (RMAX >= 2 && n2 % 2 == 0 && passes * n2 >= 4 * grid) ffn_stage<false, (RMAX >= 2 ? 2 : 1)>(a, sh, wave, lane);
    else ffn_stage<false, 1>(a, sh, wave, lane);
#ifdef MOE_FFN_TRACE
    if (threadIdx.x == 0) {
        long long *tr = reinterpret_cast<long long *>(a.part + (2 * static_cast<size_t>(kMaxGrid) - 1 - blockIdx.x) * kPartPerWg);
        tr[0] = t0; tr[1] = t1; tr[2] = t2; tr[3] = wall_clock64(); tr[4] = sh.wait_ticks;
    }
#endif
}

// ------------------------------------------------------------------ fp32 path
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, MOE_WAVE);
    return v;
}

// grid (ceil(d_e/4), T*k rows): wave w of a block computes act[r, c] for c = blockIdx.x*4 + w
__global__ __launch_bounds__(256)
void gateup_f32_kernel(const float *__restrict__ X, const float *__restrict__ W13,
                       const int32_t *__restrict__ slot_off, const int32_t *__restrict__ perm,
                       float *__restrict__ act, int C, int k, int d_h, int d_e) {
    const int r = blockIdx.y;
    if (r >= slot_off[C]) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + wave;
    if (c >= d_e) return;
    int s = 0;
    while (slot_off[s + 1] <= r) ++s;                    // slot of row r (C is small)
    const int tok = perm[r] / k;
    const float *x = X + static_cast<size_t>(tok) * d_h;
    const float *wg = W13 + (static_cast<size_t>(s) * 2 * d_e + c) * d_h;
    const float *wu = wg + static_cast<size_t>(d_e) * d_h;
    float h = 0.f, u = 0.f;
    for (int i = lane * 4; i < d_h; i += 256) {
        const float4 xv = *reinterpret_cast<const float4 *>(x + i);
        const float4 gv = *reinterpret_cast<const float4 *>(wg + i);
        const float4 uv = *reinterpret_cast<const float4 *>(wu + i);
        h += xv.x * gv.x + xv.y * gv.y + xv.z * gv.z + xv.w * gv.w;
        u += xv.x * uv.x + xv.y * uv.y + xv.z * uv.z + xv.w * uv.w;
    }
    h = wave_sum(h);
    u = wave_sum(u);
    if (lane == 0) act[static_cast<size_t>(r) * d_e + c] = h / (1.0f + expf(-h)) * u;
}

__global__ __launch_bounds__(256)
void down_f32_kernel(const float *__restrict__ act, const float *__restrict__ W2,
                     const int32_t *__restrict__ slot_off, float *__restrict__ Yp, int C, int d_h, int d_e) {
    const int r = blockIdx.y;
    if (r >= slot_off[C]) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + wave;
    if (c >= d_h) return;
    int s = 0;
    while (slot_off[s + 1] <= r) ++s;
    const float *a = act + static_cast<size_t>(r) * d_e;
    const float *wd = W2 + (static_cast<size_t>(s) * d_h + c) * d_e;
    float y = 0.f;
    for (int i = lane * 4; i < d_e; i += 256) {
        const float4 av = *reinterpret_cast<const float4 *>(a + i);
        const float4 wv = *reinterpret_cast<const float4 *>(wd + i);
        y += av.x * wv.x + av.y * wv.y + av.z * wv.z + av.w * wv.w;
    }
    y = wave_sum(y);
    if (lane == 0) Yp[static_cast<size_t>(r) * d_h + c] = y;
}

}  // namespace

extern "C" size_t moe_workspace_bytes(int T, int k, int C, int d_h, int d_e, int dtype) {
    (void)C; (void)d_h;
    if (T < 0 || k < 1 || d_e < 1) return 0;
    const size_t elt = dtype == MOE_DTYPE_F32 ? 4 : 2;
    const size_t bytes = static_cast<size_t>(T) * k * ((d_e + 63) / 64 * 64) * elt;
    return kCtrlBytes + kPartBytes + (bytes + 255) / 256 * 256 + 256;
}

extern "C" int moe_workspace_init(void *workspace_dev, size_t workspace_bytes, void *stream) {
    if (!workspace_dev || !moe::aligned(workspace_dev, 256)) return MOE_EINVAL;
    if (workspace_bytes < kCtrlBytes) return MOE_EWORKSPACE;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<int *>(workspace_dev), kCtrlInts);
    return moe::check_launch("moe_workspace_init");
}

extern "C" int moe_workspace_status(const void *workspace_dev, int *status_host) {
    if (!workspace_dev || !status_host) return MOE_EINVAL;
    int hdr[2] = {0, 0};
    hipError_t e = hipMemcpy(hdr, workspace_dev, sizeof(hdr), hipMemcpyDeviceToHost);
    if (e != hipSuccess) { moe::set_hip_error(e, "moe_workspace_status"); return MOE_EHIP; }
    *status_host = hdr[1];
    return MOE_OK;
}

extern "C" int moe_pack_weights_bf16(const void *W13_dev, const void *W2_dev, int C, int d_h, int d_e,
                                     void *W13_packed_dev, void *W2_packed_dev, void *stream) {
    if (C < 1 || d_h < 1 || d_e < 1) return MOE_EINVAL;
    if (C > MOE_MAX_SLOTS || d_h % 32 != 0 || d_e % 32 != 0) return MOE_ESHAPE;
    if (!W13_dev || !W2_dev || !W13_packed_dev || !W2_packed_dev) return MOE_EINVAL;
    if (!moe::aligned(W13_dev, 16) || !moe::aligned(W2_dev, 16) || !moe::aligned(W13_packed_dev, 16) ||
        !moe::aligned(W2_packed_dev, 16))
        return MOE_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(pack_w13_kernel, dim3(2048), dim3(256), 0, st,
                       static_cast<const uint4 *>(W13_dev), static_cast<uint4 *>(W13_packed_dev), C, d_h, d_e);
    hipLaunchKernelGGL(pack_w2_kernel, dim3(2048), dim3(256), 0, st,
                       static_cast<const uint4 *>(W2_dev), static_cast<uint4 *>(W2_packed_dev), C, d_h, d_e);
    return moe::check_launch("moe_pack_weights_bf16");
}

namespace {
// Persistent grid of the fused kernel: a multiple of the CU count that is resident at once.
// MOE_JANUS_FFN_WG_PER_CU overrides the workgroups per CU (1..limit) for tuning.
int ffn_grid_blocks(int limit_per_cu) {
    static int cus = 0;
    if (!cus) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            return 0;
        cus = n;
    }
    int per_cu = limit_per_cu;
    if (const char *e = getenv("MOE_JANUS_FFN_WG_PER_CU")) {
        const int v = atoi(e);
        if (v >= 1 && v <= limit_per_cu) per_cu = v;
    }
    const int g = cus * per_cu;
    return g < kMaxGrid ? g : kMaxGrid;
}
}  // namespace

extern "C" int moe_grouped_ffn(const void *X_dev, const void *W13_dev, const void *W2_dev,
                               int T, int k, int C, int d_h, int d_e, int dtype,
                               const int32_t *slot_off_dev, const int32_t *perm_dev,
                               float *Yp_dev, void *workspace_dev, size_t workspace_bytes, void *stream) {
    if (T < 0 || k < 1 || C < 1 || d_h < 1 || d_e < 1) return MOE_EINVAL;
    if (dtype != MOE_DTYPE_BF16 && dtype != MOE_DTYPE_F32) return MOE_EINVAL;
    if (C > MOE_MAX_SLOTS || k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (static_cast<long long>(T) * k > 0x7fffffffLL) return MOE_ESHAPE;
    if (dtype == MOE_DTYPE_BF16 && (d_h % 32 != 0 || d_e % 32 != 0)) return MOE_ESHAPE;
    if (dtype == MOE_DTYPE_F32 && (d_h % 4 != 0 || d_e % 4 != 0)) return MOE_ESHAPE;
    if (T == 0) return MOE_OK;
    if (!X_dev || !W13_dev || !W2_dev || !slot_off_dev || !perm_dev || !Yp_dev || !workspace_dev) return MOE_EINVAL;
    if (!moe::aligned(X_dev, 16) || !moe::aligned(W13_dev, 16) || !moe::aligned(W2_dev, 16) ||
        !moe::aligned(Yp_dev, 16) || !moe::aligned(workspace_dev, 256) || !moe::aligned(slot_off_dev, 4) ||
        !moe::aligned(perm_dev, 4))
        return MOE_EINVAL;
    if (workspace_bytes < moe_workspace_bytes(T, k, C, d_h, d_e, dtype)) return MOE_EWORKSPACE;
    if (dtype == MOE_DTYPE_BF16) {
        // the kernel numbers its work (passes x units x quads of 4 K-steps) in 32 bits
        const long long passes = static_cast<long long>(T) * k / 16 + C;
        const long long q1 = passes * (d_e / 16) * ((d_h / 32 + 3) / 4), q2 = passes * (d_h / 32) * ((d_e / 32 + 3) / 4);
        if (q1 > 0x3fffffffLL || q2 > 0x3fffffffLL) return MOE_ESHAPE;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace_dev);
    if (dtype == MOE_DTYPE_BF16) {
        static const bool use_stream = getenv("MOE_JANUS_FFN_FUSED") == nullptr;
        if (use_stream) {
            moe::launch_ffn_stream(X_dev, W13_dev, W2_dev, T, k, C, d_h, d_e, slot_off_dev, perm_dev,
                                   reinterpret_cast<uint16_t *>(ws + kCtrlBytes + kPartBytes), (d_e + 63) / 64 * 64,
                                   Yp_dev, st);
            return moe::check_launch("moe_grouped_ffn");
        }
        const int blocks = ffn_grid_blocks(kFfnWgPerCu);
        if (blocks < 1) { moe::set_hip_error(hipErrorInvalidDevice, "moe_grouped_ffn/device query"); return MOE_EHIP; }
        FfnArgs a;
        a.X = static_cast<const uint16_t *>(X_dev);
        a.W13p = static_cast<const bf16x8 *>(W13_dev);
        a.W2p = static_cast<const bf16x8 *>(W2_dev);
        a.slot_off = slot_off_dev;
        a.perm = perm_dev;
        a.ctrl = reinterpret_cast<int *>(ws);
        a.part = reinterpret_cast<f32x4 *>(ws + kCtrlBytes);
        a.act = reinterpret_cast<uint16_t *>(ws + kCtrlBytes + kPartBytes);
        a.Yp = Yp_dev;
        a.k = k; a.C = C; a.d_h = d_h; a.d_e = d_e;
        a.act_stride = (d_e + 63) / 64 * 64;
        a.spin_limit = 1 << 21;
        hipLaunchKernelGGL(ffn_fused_kernel, dim3(blocks), dim3(kFfnThreads), 0, st, a);
    } else {
        // one grid row per possible request row; rows >= n_local leave at once
        const long long rows = static_cast<long long>(T) * k;
        if (rows > 65535) return MOE_ESHAPE;
        float *act = reinterpret_cast<float *>(ws + kCtrlBytes + kPartBytes);
        hipLaunchKernelGGL(gateup_f32_kernel, dim3((d_e + 3) / 4, rows), dim3(256), 0, st,
                           static_cast<const float *>(X_dev), static_cast<const float *>(W13_dev),
                           slot_off_dev, perm_dev, act, C, k, d_h, d_e);
        hipLaunchKernelGGL(down_f32_kernel, dim3((d_h + 3) / 4, rows), dim3(256), 0, st,
                           act, static_cast<const float *>(W2_dev), slot_off_dev, Yp_dev, C, d_h, d_e);
    }
    return moe::check_launch("moe_grouped_ffn");
}
