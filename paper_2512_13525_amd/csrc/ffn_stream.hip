// a5, bf16 path: the grouped expert FFN (gate/up + SiLU*up, then down) as oversubscribed streaming
// workgroups.
//
// Janus Sec. 2.2: at decode sizes an expert is two skinny GEMMs whose cost is the weight bytes
// streamed from HBM, so the layer's latency follows the number of activated experts.  The work
// of a stage is cut into items = (block of up to 32 or 64 request rows of one slot) x (tile of 16
// gate+up channels in stage 1, 32 output channels in stage 2); one workgroup per item, in plain
// grid order, dispatched by the hardware.  Slots without requests own no item: their weights are
// never read.  Nothing about the activated set is known on the host, so the grid is sized for
// the largest possible number of blocks; the dispatch step leaves the list of blocks in device
// memory, a workgroup reads its entry with two scalar loads, and workgroups past the last block
// leave at once.
//
// The 4 wavefronts of a workgroup split the K dimension of the tile round-robin in super-steps
// of 64 columns and meet in LDS once, at the end (fixed summation order: results are
// reproducible).  Per super-step a wavefront reads 4 KiB of weights (packed MFMA A-operand
// images, fully coalesced 128-bit loads, two super-steps ahead) and the token rows (the B operand,
// from L2).  In stage 1 those are gathered rows of X: one 128-byte line of each row, one super-step
// ahead, turned into the MFMA layout through a wave-private LDS tile.  Stage 1 writes `act` as
// B-operand images, so stage 2 reads its token fragments like the weights, straight into
// registers and as far ahead.
//
// Every further streaming block of a slot streams the expert's tiles again.  When a batch has enough
// slots with more than 64 requests (wide_on below), those slots are computed as tiled GEMMs over
// blocks of 64 rows by workgroups of the same launch instead (wide_item): a workgroup takes four
// channel tiles through the whole K dimension, shares the token rows of the block between them
// through LDS, and the blocks of a slot are dealt to the workgroups so that they find the
// expert's tiles in their XCD's L2 (run_wide).
//
// Both stages run in ONE launch: the stage-2 workgroups have the higher ids, so the hardware
// starts them only after every stage-1 workgroup has been started, and they fill the compute
// units that the tail of stage 1 leaves idle.  A stage-2 workgroup first puts its weight loads in
// flight and then waits until the 16-channel tiles of its block of `act` rows are all written: a
// counter per block in the workspace is bumped by each stage-1 workgroup once its stores are
// acknowledged; the workgroup that completes the count raises the block's ready flags, which the
// stage-2 workgroups poll (bounded; on an overrun the workgroup raises the workspace's error word,
// writes NaN rows instead of results and leaves, so every wave reaches the end of the kernel).  The 8 XCDs do not share an
// L2: `act` is written with agent-scope (write-through) stores, every 128-byte line of it has one
// writing workgroup, and no workgroup reads a line before its block is ready, so plain loads see
// the data; counters and flags are agent-scope atomics.  The last stage-2 workgroup of a block to
// get through the wait clears the block's control lines for the next call.
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kDepthA = 2;              // super-steps of weight loads each wavefront keeps in flight
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / MOE_WAVE;
// A launch is compiled for blocks of TT token tiles of 16 rows (TT = 2 or 4: blocks of 32 or 64
// request rows); one 16-channel tile of a block of act takes TT*16 rows x 32 bytes.

// Control region of the workspace (ints): [1] error word; block j owns the 8 lines of 128 bytes
// at int offset (j+1)*kCtrlBlockInts: line 0 = {stage-1 tiles done, stage-2 workgroups through},
// lines 1..7 = copies of the block's ready flag (same-address accesses from many workgroups
// serialise in the memory system, so the pollers are spread over the copies).
constexpr int kCtrlLineInts = 32;
constexpr int kCtrlCopies = 7;
constexpr int kCtrlBlockInts = (1 + kCtrlCopies) * kCtrlLineInts;
constexpr int kMaxItems = static_cast<int>(moe::kFfnCtrlBytes / 4) / kCtrlBlockInts - 1;

struct StageArgs {
    const uint16_t *B;                   // token operand: X (stage 1, rows through perm) or act (stage 2, blocks)
    const char *Wp;                      // packed weights: [C][tiles][KS][2][64] fragments of 16 bytes
    int tiles, items, tiles_pad, KS;     // items = workgroups per block (stage 2: one per pair of tiles); tiles_pad = items rounded up to a multiple of 8
    int b_stride;                        // elements between rows of X (stage 1)
    int out_stride;                      // elements between rows of Yp (stage 2)
};

struct StreamArgs {
    StageArgs s[2];
    const int32_t *blocks;               // work list written by the dispatch step
    const int32_t *perm;
    uint16_t *act;                       // stage-1 output
    float *Yp;                           // stage-2 output
    int *ctrl;
    int k, C;
    int spin_limit;
    uint32_t act_block_bytes;            // bytes of `act` per entry of the work list: R rows x d_e rounded up to 64 channels
    int has_gemm;                        // the batch is large enough for the separate tiled-GEMM launches (common.h)
};

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// The weights of a slot with a single block are read exactly once: they are loaded with the
// streaming hint (STREAM), so that on their way through an L2 they do not push out the token rows,
// which every tile of a block reads again (7 MB of rows against a 4 MB L2 at d_h = 7168, T = 512:
// 237 -> 227 us for that launch).  The blocks of a slot with several share their tiles through L2
// and keep the plain loads (with the hint on those too, all-slot batches of 128 to 512 tokens
// were 20 % slower).
template <bool STREAM>
__device__ __forceinline__ bf16x8 load_weights(const char *p) {
    if constexpr (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const bf16x8 *>(p));
    else return *reinterpret_cast<const bf16x8 *>(p);
}

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + __expf(-g)) * u; }

// Workgroup barrier for LDS exchange only: waits for this wavefront's LDS traffic, not for its
// global loads (prefetched weights stay in flight across it).
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Split-K reduction over the 4 wavefronts in LDS (fixed order), then the epilogue: SiLU(gate)*up
// rounded once to bf16 (stage 1, agent-scope stores) or the fp32 partial output rows (stage 2).
template <bool STAGE1, int NT, int TT>
__device__ __forceinline__ void reduce_store(const StreamArgs &a, const StageArgs &g,
                                             f32x4 (*red)[2][TT][MOE_WAVE], f32x4 (&acc)[2][NT],
                                             int item_id, int brow, int tile, int row0, int row_end, int wave, int lane) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int t = 0; t < NT; ++t) red[wave][h][t][lane] = acc[h][t];
    __syncthreads();
    if (STAGE1) {
        // lane-slot (t, l) holds gate/up channels tile*16 + (l/16)*4 .. +3 of token row0 + t*16 + l%16
        for (int item = threadIdx.x; item < NT * MOE_WAVE; item += kThreads) {
            const int t = item / MOE_WAVE, l = item % MOE_WAVE;
            f32x4 gt = red[0][0][t][l], up = red[0][1][t][l];
#pragma unroll
            for (int wv = 1; wv < kWaves; ++wv) { gt += red[wv][0][t][l]; up += red[wv][1][t][l]; }
            const int r = row0 + t * 16 + (l & 15);
            if (r < row_end) {
                const uint64_t o = static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(gt[0], up[0]))) |
                                   static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(gt[1], up[1]))) << 16 |
                                   static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(gt[2], up[2]))) << 32 |
                                   static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(gt[3], up[3]))) << 48;
                // act block of this item: [K-step of stage 2][token tile][64 lanes][16 B], the register image of
                // the MFMA B operand (lane: row % 16, channels (lane / 16) * 8 .. + 7 of the K-step's 32); this
                // tile is half a K-step, and every 128-byte line of the image has one writing workgroup
                const int fl = (l & 15) + 16 * ((tile & 1) * 2 + (l >> 5));
                uint64_t *dst = reinterpret_cast<uint64_t *>(
                    reinterpret_cast<char *>(a.act) + static_cast<size_t>(item_id) * a.act_block_bytes +
                    (static_cast<size_t>(tile >> 1) * TT + (brow >> 4) + t) * 1024 +
                    fl * 16 + ((l >> 4) & 1) * 8);
                __hip_atomic_store(dst, o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    } else {
        // lane-slot (h, t, l) holds output channels tile*32 + h*16 + (l/16)*4 .. +3
        for (int item = threadIdx.x; item < 2 * NT * MOE_WAVE; item += kThreads) {
            const int h = item / (NT * MOE_WAVE), t = item / MOE_WAVE % NT, l = item % MOE_WAVE;
            f32x4 y = red[0][h][t][l];
#pragma unroll
            for (int wv = 1; wv < kWaves; ++wv) y += red[wv][h][t][l];
            const int r = row0 + t * 16 + (l & 15);
            if (r < row_end)
                *reinterpret_cast<f32x4 *>(a.Yp + static_cast<size_t>(r) * g.out_stride + tile * 32 + h * 16 + (l >> 4) * 4) = y;
        }
    }
}

// Stage 2 of a block may read `act` only when all stage-1 tiles of the block are written: the
// stage-1 workgroup that completes the count raises the block's ready flags.  Called by the whole
// workgroup; thread 0 polls one copy of the flag.  The second counter of the block counts the
// stage-2 workgroups that got through: the last one clears the block's control lines for the
// next call.  Returns false when the bounded wait ran out: the status word gets bit 0, the
// block's control lines are left as they are (a late stage-1 tile may still bump them, so the
// region needs moe_workspace_init before the next call), and the caller must not read `act`.
__device__ __forceinline__ bool wait_block_ready(const StreamArgs &a, int *s_ok, int item, int tile, int n_readers) {
    if (threadIdx.x == 0) {
        int *blk = a.ctrl + (item + 1) * kCtrlBlockInts;
        const int *flag = blk + (1 + tile % kCtrlCopies) * kCtrlLineInts;
        // header word 2: a spin limit for this workspace (tests of the overrun path); 0 = the default
        const int lim_ws = a.ctrl[moe::kCtrlSpinLimit];
        const int limit = lim_ws > 0 ? lim_ws : a.spin_limit;
        int spins = 0, ok = 1;
        while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
            if (++spins > limit) {
                __hip_atomic_fetch_or(a.ctrl + moe::kCtrlStatus, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
        if (ok && __hip_atomic_fetch_add(blk + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_readers - 1) {
            __hip_atomic_store(blk, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(blk + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int c = 1; c <= kCtrlCopies; ++c)
                __hip_atomic_store(blk + c * kCtrlLineInts, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        *s_ok = ok;
    }
    lds_barrier();
    return *s_ok != 0;
}

// The rows of a stage-2 item whose block never became ready: quiet NaNs, so that the combine
// propagates them and nobody mistakes the rows for results.
__device__ __forceinline__ void store_nan_rows(const StreamArgs &a, const StageArgs &g, int tile, int row0, int n_rows) {
    const float qnan = __uint_as_float(0x7fc00000u);
    const f32x4 v = {qnan, qnan, qnan, qnan};
    for (int i = threadIdx.x; i < n_rows * 8; i += kThreads)
        *reinterpret_cast<f32x4 *>(a.Yp + static_cast<size_t>(row0 + i / 8) * g.out_stride + tile * 32 + (i % 8) * 4) = v;
}

// One stage-1 item with an even number of K-steps.  A super-step is two K-steps = 64 columns = one
// 128-byte line of every token row.
// A token load instruction fetches whole lines (lane l: row l/8, 16-byte chunk l%8), so no line
// is requested twice and none by halves; the MFMA layout (lane l: row l%16, 16-byte chunk 4*step + l/16) is produced by a
// round trip through a wave-private 2 KiB LDS tile per 16 rows (chunks XOR-swizzled by row so
// that both the row-major writes and the column-wise reads spread over the banks).  NH = number
// of 8-row halves that hold requests (rows past the end repeat the last row; halves past it are
// not loaded and leave unspecified values in token columns whose results are never stored).
template <int NH, int TT, bool STREAM>
__device__ __forceinline__ void stream_item_lines(const StreamArgs &a, const StageArgs &g, char *lds,
                                                  const char *w, int item, int tile, int row0, int row_end,
                                                  int wave, int lane) {
    asm volatile("" : "+v"(lane));                             // see wide_item
    constexpr int NT = (NH + 1) / 2;
    constexpr int D = kDepthA;
    f32x4 (*red)[2][TT][MOE_WAVE] = reinterpret_cast<f32x4 (*)[2][TT][MOE_WAVE]>(lds);
    char *stg = lds + wave * (TT * 2048);
    const uint32_t aoff = lane * 16;
    // token rows: wave-uniform base (advanced per super-step) + constant 32-bit per-lane byte offset
    uint32_t boff[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        int r = row0 + h * 8 + (lane >> 3);
        r = r < row_end ? r : row_end - 1;
        boff[h] = static_cast<uint32_t>(a.perm[r] / a.k) * static_cast<uint32_t>(g.b_stride) * 2 + (lane & 7) * 16;
    }
    // LDS: row R of a tile at R*128, its 16-byte chunk c at ((c ^ ((R >> 1) & 7)) * 16): the 16 rows a
    // fragment read touches fall into 16 different bank groups.  wr_lds[p]: rows of an even / odd half.
    const uint32_t wr_lds[2] = {static_cast<uint32_t>(((lane >> 3) * 128) + (((lane & 7) ^ (lane >> 4)) * 16)),
                                static_cast<uint32_t>(((lane >> 3) * 128) + (((lane & 7) ^ (4 + (lane >> 4))) * 16))};
    const uint32_t rd_row = (lane & 15) * 128, rd_sw = (lane >> 1) & 7, rd_g = lane >> 4;
    const char *bbase = reinterpret_cast<const char *>(g.B);
    constexpr int kBStep = 128;                                  // bytes a super-step advances a token row
    const int n = (g.KS / 2 - wave + kWaves - 1) / kWaves;      // super-steps wave, wave+4, ... of this wavefront
    f32x4 acc[2][NT];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[h][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Weights run D super-steps ahead (ring wr); the token rows DB super-steps: the loads of
    // super-step q+DB are issued in iteration q *before* the weights of q+D.  Loads return in order,
    // so waiting for the token rows of the next super-step also waits for every older weight load:
    // with DB = 1 only the newest super-step of weights stays in flight across that wait, with
    // DB = 2 (where the registers allow it: blocks of up to 16 rows, 32 in the 64-row kernel) two do.  The steady-state
    // loop has no branch, so the compiler counts outstanding loads exactly; before and after it
    // loads are only issued for super-steps that exist.
    constexpr int DB = (NH <= 4) ? D : 1;                        // D: the two rings share their positions
    bf16x8 wr[D][2][2];
    bf16x8 br[DB][NH];
    const int last = n > 0 ? n - 1 : 0;
    // Workgroups start their K loop at different places (and wrap around) so that they do not
    // march through equally aligned tiles in lockstep.
    const int rot = n > 0 ? static_cast<int>(static_cast<unsigned>(tile) % static_cast<unsigned>(n)) : 0;
#define MOE_STEP_INDEX(step)                                                                     \
        const int q_ = (step);                                                                   \
        int r_ = (q_ < last ? q_ : last) + rot;                                                  \
        r_ = r_ >= n ? r_ - n : r_;                                                              \
        const int s_ = wave + kWaves * r_;
#define MOE_LOAD_A(d, step)                                                                      \
    do {                                                                                         \
        MOE_STEP_INDEX(step)                                                                     \
        const char *ws_ = w + static_cast<size_t>(s_) * 4096;                                    \
        _Pragma("unroll") for (int ss = 0; ss < 2; ++ss) {                                       \
            wr[d][ss][0] = load_weights<STREAM>(ws_ + ss * 2048 + aoff);                        \
            wr[d][ss][1] = load_weights<STREAM>(ws_ + ss * 2048 + 1024 + aoff);                 \
        }                                                                                        \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
#define MOE_LOAD_B(d, step)                                                                      \
    do {                                                                                         \
        MOE_STEP_INDEX(step)                                                                     \
        const char *bs_ = bbase + static_cast<size_t>(s_) * kBStep;                              \
        _Pragma("unroll") for (int h = 0; h < NH; ++h)                                           \
            br[(d) % DB][h] = *reinterpret_cast<const bf16x8 *>(bs_ + boff[h]);                  \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
#define MOE_STAGE_B(d)                                                                           \
    do {                                                                                         \
        _Pragma("unroll") for (int h = 0; h < NH; ++h)                                           \
            *reinterpret_cast<bf16x8 *>(stg + (h / 2) * 2048 + (h % 2) * 1024 + wr_lds[h % 2]) = br[(d) % DB][h]; \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
#define MOE_MMA_STEP(d)                                                                          \
    do {                                                                                         \
        _Pragma("unroll") for (int ss = 0; ss < 2; ++ss)                                         \
            _Pragma("unroll") for (int t = 0; t < NT; ++t) {                                     \
                const bf16x8 bf_ = *reinterpret_cast<const bf16x8 *>(                            \
                    stg + t * 2048 + rd_row + (((4 * ss + rd_g) ^ rd_sw) * 16));                 \
                acc[0][t] = mfma16(wr[d][ss][0], bf_, acc[0][t]);                                \
                acc[1][t] = mfma16(wr[d][ss][1], bf_, acc[1][t]);                                \
            }                                                                                    \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
    if (n > 0) {
        // issue order of the first loads: tokens of a super-step before its weights
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (d < DB && d < n) MOE_LOAD_B(d, d);
            if (d < n) MOE_LOAD_A(d, d);
        }
        int i = 0;
        for (; i + 2 * D <= n; i += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                MOE_STAGE_B(d);
                MOE_LOAD_B(d + DB, i + d + DB);
                MOE_MMA_STEP(d);
                MOE_LOAD_A(d, i + d + D);
            }
        }
        const int rem = n - i;                                   // 1 .. 2*D-1 super-steps left
        // the last 1 .. 2*D-1 super-steps: only those that exist are loaded, staged and multiplied
        // (wave-uniform conditions)
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (d < rem) MOE_STAGE_B(d);
            if (d + DB < rem) MOE_LOAD_B(d + DB, i + d + DB);
            if (d < rem) MOE_MMA_STEP(d);
            if (d < D - 1 && d + D < rem) MOE_LOAD_A(d, i + d + D);
        }
#pragma unroll
        for (int d = 0; d < D - 1; ++d) {
            if (D + d < rem) {
                MOE_STAGE_B(D + d);
                MOE_MMA_STEP(d);
            }
        }
    }
#undef MOE_STEP_INDEX
#undef MOE_LOAD_A
#undef MOE_LOAD_B
#undef MOE_STAGE_B
#undef MOE_MMA_STEP
    __syncthreads();                                             // the staging tiles are reused for the reduction
    reduce_store<true, NT, TT>(a, g, red, acc, item, 0, tile, row0, row_end, wave, lane);
}

// One stage-1 item with an odd number of K-steps (shapes that are multiples of 32 but not of 64): single
// K-steps, token rows read 64 bytes at a time straight into the MFMA layout (lane l: row l%16,
// 16 bytes at (l/16)*16), four steps of weights and tokens in flight.
template <int NT, int TT>
__device__ __forceinline__ void stream_item_steps(const StreamArgs &a, const StageArgs &g, char *lds,
                                                  const char *w, int item, int brow, int tile, int row0, int row_end,
                                                  int wave, int lane) {
    asm volatile("" : "+v"(lane));                             // see wide_item
    constexpr int D = 2 * kDepthA;
    f32x4 (*red)[2][TT][MOE_WAVE] = reinterpret_cast<f32x4 (*)[2][TT][MOE_WAVE]>(lds);
    const uint32_t aoff = lane * 16;
    uint32_t boff[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int r = row0 + t * 16 + (lane & 15);
        r = r < row_end ? r : row_end - 1;
        boff[t] = (static_cast<uint32_t>(a.perm[r] / a.k) * static_cast<uint32_t>(g.b_stride) + (lane >> 4) * 8) * 2;
    }
    const char *bbase = reinterpret_cast<const char *>(g.B);
    constexpr int kBStep = 64;                                   // bytes a K-step advances a token row
    const int n = (g.KS - wave + kWaves - 1) / kWaves;          // K-steps wave, wave+4, ... of this wavefront
    f32x4 acc[2][NT];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[h][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (n > 0) {
        bf16x8 wr[D][2], br[D][NT];
        const int last = n - 1;
        const int rot = static_cast<int>(static_cast<unsigned>(tile) % static_cast<unsigned>(n));
#define MOE_LOAD_STEP(d, step)                                                                   \
        do {                                                                                     \
            const int q_ = (step);                                                               \
            int r_ = (q_ < last ? q_ : last) + rot;                                              \
            r_ = r_ >= n ? r_ - n : r_;                                                          \
            const int s_ = wave + kWaves * r_;                                                   \
            const char *ws_ = w + static_cast<size_t>(s_) * 2048;                                \
            const char *bs_ = bbase + static_cast<size_t>(s_) * kBStep;                            \
            wr[d][0] = load_weights<false>(ws_ + aoff);                                          \
            wr[d][1] = load_weights<false>(ws_ + 1024 + aoff);                                   \
            _Pragma("unroll") for (int t = 0; t < NT; ++t)                                       \
                br[d][t] = *reinterpret_cast<const bf16x8 *>(bs_ + boff[t]);                     \
            asm volatile("" ::: "memory");                                                       \
        } while (0)
#define MOE_MMA_STEP(d)                                                                          \
        do {                                                                                     \
            _Pragma("unroll") for (int t = 0; t < NT; ++t) {                                     \
                acc[0][t] = mfma16(wr[d][0], br[d][t], acc[0][t]);                               \
                acc[1][t] = mfma16(wr[d][1], br[d][t], acc[1][t]);                               \
            }                                                                                    \
        } while (0)
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (d < n) MOE_LOAD_STEP(d, d);
        int i = 0;
        for (; i + 2 * D <= n; i += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                MOE_MMA_STEP(d);
                MOE_LOAD_STEP(d, i + d + D);
            }
        }
        const int rem = n - i;                                   // 1 .. 2*D-1 steps left
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (d < rem) MOE_MMA_STEP(d);
            if (d < D - 1 && d + D < rem) MOE_LOAD_STEP(d, i + d + D);
        }
#pragma unroll
        for (int d = 0; d < D - 1; ++d)
            if (D + d < rem) MOE_MMA_STEP(d);
#undef MOE_LOAD_STEP
#undef MOE_MMA_STEP
    }
    reduce_store<true, NT, TT>(a, g, red, acc, item, brow, tile, row0, row_end, wave, lane);
}

// Stage 2 of one item.  Stage 1 leaves the block's rows of `act` as MFMA B-operand images, so a
// token fragment is one coalesced 1 KiB load straight into registers, like a weight fragment, with
// no LDS on the way.  A step is U K-steps (U = 2, 4 KiB of contiguous weights, when the number of
// K-steps is even and the token tiles leave room in the registers); the steps go round-robin over
// the wavefronts, 4 / U or 3 of them in flight for both operands, the weights issued before the
// wait for the block (they do not depend on stage 1).
// NW = 2: the item is a pair of adjacent tiles (64 output channels; their weights follow each other in
// the packed layout) multiplied with the same token fragments: half as many items and `act`
// loads per block, twice the weight bytes in flight per workgroup.  Blocks of up to 16 rows (32
// in the 64-row launch) have the registers for it.  n_readers: calls of this function per block.
template <int NT, int TT, int U, bool STREAM, int NW>
__device__ __forceinline__ void stream_item_down(const StreamArgs &a, const StageArgs &g, char *lds, int *s_ok,
                                                 const char *w, int item, int tile, int n_readers, int row0, int row_end,
                                                 int wave, int lane) {
    asm volatile("" : "+v"(lane));                             // see wide_item
    constexpr int D = U == 2 ? 2 : NT > 2 ? 3 : 4;               // steps in flight that fit the registers
    constexpr int F = 2 * NW;                                    // weight fragments per K-step
    const size_t w_tile = static_cast<size_t>(g.KS) * 2048;     // bytes between the tiles of the pair
    f32x4 (*red)[2][TT][MOE_WAVE] = reinterpret_cast<f32x4 (*)[2][TT][MOE_WAVE]>(lds);
    const uint32_t aoff = lane * 16;
    const char *bbase = reinterpret_cast<const char *>(g.B) + static_cast<size_t>(item) * a.act_block_bytes + aoff;
    const int n = (g.KS / U - wave + kWaves - 1) / kWaves;      // steps wave, wave+4, ... of this wavefront
    f32x4 acc[F][NT];
#pragma unroll
    for (int h = 0; h < F; ++h)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[h][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    bf16x8 wr[D][U][F], br[D][U][NT];
    const int last = n > 0 ? n - 1 : 0;
    const int rot = n > 0 ? static_cast<int>(static_cast<unsigned>(tile) % static_cast<unsigned>(n)) : 0;
#define MOE_STEP_INDEX(step)                                                                     \
        const int q_ = (step);                                                                   \
        int r_ = (q_ < last ? q_ : last) + rot;                                                  \
        r_ = r_ >= n ? r_ - n : r_;                                                              \
        const int s_ = wave + kWaves * r_;
#define MOE_LOAD_W(d, step)                                                                      \
    do {                                                                                         \
        MOE_STEP_INDEX(step)                                                                     \
        const char *ws_ = w + static_cast<size_t>(s_) * (U * 2048) + aoff;                       \
        _Pragma("unroll") for (int nw = 0; nw < NW; ++nw)                                        \
            _Pragma("unroll") for (int u = 0; u < U; ++u) {                                      \
                wr[d][u][2 * nw] = load_weights<STREAM>(ws_ + nw * w_tile + u * 2048);          \
                wr[d][u][2 * nw + 1] = load_weights<STREAM>(ws_ + nw * w_tile + u * 2048 + 1024); \
            }                                                                                    \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
#define MOE_LOAD_T(d, step)                                                                      \
    do {                                                                                         \
        MOE_STEP_INDEX(step)                                                                     \
        const char *bs_ = bbase + static_cast<size_t>(s_) * (U * TT * 1024);                     \
        _Pragma("unroll") for (int u = 0; u < U; ++u)                                            \
            _Pragma("unroll") for (int t = 0; t < NT; ++t)                                       \
                br[d][u][t] = *reinterpret_cast<const bf16x8 *>(bs_ + (u * TT + t) * 1024);      \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
#define MOE_MMA_STEP(d)                                                                          \
    do {                                                                                         \
        _Pragma("unroll") for (int u = 0; u < U; ++u)                                            \
            _Pragma("unroll") for (int t = 0; t < NT; ++t)                                       \
                _Pragma("unroll") for (int f = 0; f < F; ++f)                                    \
                    acc[f][t] = mfma16(wr[d][u][f], br[d][u][t], acc[f][t]);                     \
    } while (0)
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < n) MOE_LOAD_W(d, d);
    if (!wait_block_ready(a, s_ok, item, tile, n_readers)) {
        const int m_ = row_end - row0;
#pragma unroll
        for (int nw = 0; nw < NW; ++nw) store_nan_rows(a, g, tile + nw, row0, m_ < TT * 16 ? m_ : TT * 16);
        return;
    }
    if (n > 0) {
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (d < n) MOE_LOAD_T(d, d);
        int i = 0;
        for (; i + 2 * D <= n; i += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                MOE_MMA_STEP(d);
                MOE_LOAD_W(d, i + d + D);
                MOE_LOAD_T(d, i + d + D);
            }
        }
        const int rem = n - i;                                   // 1 .. 2*D-1 steps left
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (d < rem) MOE_MMA_STEP(d);
            if (d < D - 1 && d + D < rem) { MOE_LOAD_W(d, i + d + D); MOE_LOAD_T(d, i + d + D); }
        }
#pragma unroll
        for (int d = 0; d < D - 1; ++d)
            if (D + d < rem) MOE_MMA_STEP(d);
    }
#undef MOE_STEP_INDEX
#undef MOE_LOAD_W
#undef MOE_LOAD_T
#undef MOE_MMA_STEP
#pragma unroll
    for (int nw = 0; nw < NW; ++nw) {
        if (nw) __syncthreads();                                 // the reduction buffer is reused
        f32x4 part[2][NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) { part[0][t] = acc[2 * nw][t]; part[1][t] = acc[2 * nw + 1][t]; }
        reduce_store<false, NT, TT>(a, g, red, part, item, 0, tile + nw, row0, row_end, wave, lane);
    }
}

// ---------------------------------------------------------------------------------------------
// Slots with more requests than one block holds ("wide" slots): blocks of up to RT*16 rows as tiled
// GEMMs inside the same launch.  The streaming items above re-read a tile's weights for every block
// of rows and every item gathers its token rows again; here a workgroup computes RT*16 rows x 4
// packed weight tiles (64 channels of SiLU(gate)*up in stage 1, 128 output channels in stage 2),
// so the weights are fetched once per RT*16 rows and the token rows once per 4 tiles.
//
// Each of the 4 wavefronts owns one packed tile (two MFMA A fragments per K-step, read straight from
// global memory: the packed layout is the register image) and all rows: RT row tiles x 2
// accumulators.  Gate and up of a channel live in the same lane, so stage 1 needs no exchange between
// wavefronts, and a wavefront runs the whole K dimension (no split-K, no reduction).  The token rows
// (the B operand, shared by the 4 wavefronts) go through LDS: per K-tile of 64 columns the workgroup
// reads one 128-byte line of each row with whole-line loads (8 rows per instruction) into a
// double-buffered, XOR-swizzled tile, from which every wavefront reads the MFMA layout.  One
// barrier per K-tile; two K-tiles of both operands are in flight in registers.
//
// A wide block is led by the list entry whose first row is a multiple of RT*16 rows into the slot;
// the block's workgroups are the first ceil(tiles/4) ids of that entry (the others, and all ids of
// the slot's other entries, leave).  The intermediate of a wide block lives in the `act` region of
// its leading entry as [K-tile of stage 2 = 64 channels][row][128 bytes]: every 128-byte line has one
// writing workgroup, and stage 2 reads a K-tile of all rows as one contiguous run.  The hand-off is
// the one of the streaming items: counter and flags of the leading entry.
template <bool STAGE1, int RT>
__device__ __forceinline__ void wide_item(const StreamArgs &a, const StageArgs &g, char *lds, int *s_ok,
                                          int item, int group, int n_groups, int slot, int row0, int m) {
    constexpr int kRing = 2;                                         // K-tiles of both operands in flight
    constexpr bool STREAM = false;                                   // a wide slot has several blocks: they share the tiles through L2
    constexpr int kPieces = RT * 16 * 8;                             // 16-byte pieces of one K-tile of the token tile
    constexpr int kLoadsB = (kPieces + kThreads - 1) / kThreads;
    constexpr int kBufBytes = RT * 16 * 128;
    // an opaque copy of the thread id: nothing derived from it is shared with (and hoisted above) the
    // other kinds of items, whose paths would then carry it in registers
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int wave = __builtin_amdgcn_readfirstlane(tid / MOE_WAVE), lane = tid % MOE_WAVE;
    int pt = group * kWaves + wave;
    const bool pt_ok = pt < g.tiles;
    pt = pt_ok ? pt : g.tiles - 1;
    const char *w = g.Wp + (static_cast<size_t>(slot) * g.tiles + pt) * g.KS * 2048 + lane * 16;
    const int rows_pad = (m + 15) & ~15;
    char *act_blk = reinterpret_cast<char *>(a.act) + static_cast<size_t>(item) * a.act_block_bytes;

    if constexpr (!STAGE1) {
        if (!wait_block_ready(a, s_ok, item, group, n_groups)) {
            const float qnan = __uint_as_float(0x7fc00000u);
            const f32x4 v = {qnan, qnan, qnan, qnan};
            const int c0 = group * 128, nc = (g.tiles * 32 - c0 < 128 ? g.tiles * 32 - c0 : 128) / 4;
            for (int i = tid; i < m * nc; i += kThreads)
                *reinterpret_cast<f32x4 *>(a.Yp + static_cast<size_t>(row0 + i / nc) * g.out_stride + c0 + (i % nc) * 4) = v;
            return;
        }
    }

    // token rows this thread fetches: piece q*256 + tid = row (q*32 + tid/8), 16-byte chunk tid%8 of the line
    const bool loader = kPieces >= kThreads || tid < kPieces;
    const char *bp[kLoadsB];
    const size_t kt_stride = STAGE1 ? 128 : static_cast<size_t>(rows_pad) * 128;   // bytes a K-tile advances a row
#pragma unroll
    for (int q = 0; q < kLoadsB; ++q) {
        int r = q * (kThreads / 8) + (tid >> 3);
        r = r < m ? r : m - 1;
        if constexpr (STAGE1)
            bp[q] = reinterpret_cast<const char *>(g.B) +
                    static_cast<size_t>(a.perm[row0 + r] / a.k) * static_cast<uint32_t>(g.b_stride) * 2 + (tid & 7) * 16;
        else
            bp[q] = act_blk + static_cast<size_t>(r) * 128 + (tid & 7) * 16;
    }
    // LDS: row R at R*128, its 16-byte chunk c at ((c ^ ((R >> 1) & 7)) * 16): the 16 rows that one
    // fragment read touches then fall into 16 different bank groups (rows R and R+8 share R & 7)
    const uint32_t wr_lds = (tid >> 3) * 128 + (((tid & 7) ^ ((tid >> 4) & 7)) * 16);
    const uint32_t rd_row = (lane & 15) * 128, rd_sw = (lane >> 1) & 7, rd_g = lane >> 4;

    const int NKT = (g.KS + 1) >> 1;                                 // K-tiles of two K-steps (the last may hold one); >= 1
    f32x4 acc[RT][2];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) { acc[rt][0] = f32x4{0.f, 0.f, 0.f, 0.f}; acc[rt][1] = acc[rt][0]; }
    // K-tile i uses register set i % kRing and LDS buffer i % 2; loads past the last K-tile fetch the
    // last one again, so the steady-state loop has no branch around a load and the compiler counts
    // outstanding loads exactly.
    bf16x8 breg[kRing][kLoadsB];
    bf16x8 areg[kRing][2][2];                                        // [set][K-step of the tile][fragment]
    const int last = NKT - 1;

    // K-tile j: columns 64*j .. 64*j+63.  With an odd number of K-steps the last tile has only its
    // first half: its second K-step repeats the first (never multiplied) and chunks 4..7 of the
    // line, which lie past the row (stage 1) or were never written (stage 2), repeat chunks 0..3.
#define MOE_WIDE_LOAD_A(set, j)                                                                  \
    do {                                                                                         \
        const int j_ = (j) < last ? (j) : last;                                                  \
        const int s0_ = 2 * j_, s1_ = 2 * j_ + 1 < g.KS ? 2 * j_ + 1 : 2 * j_;                   \
        areg[set][0][0] = load_weights<STREAM>(w + static_cast<size_t>(s0_) * 2048);            \
        areg[set][0][1] = load_weights<STREAM>(w + static_cast<size_t>(s0_) * 2048 + 1024);     \
        areg[set][1][0] = load_weights<STREAM>(w + static_cast<size_t>(s1_) * 2048);            \
        areg[set][1][1] = load_weights<STREAM>(w + static_cast<size_t>(s1_) * 2048 + 1024);     \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
#define MOE_WIDE_LOAD_B(set, j)                                                                  \
    do {                                                                                         \
        const int j_ = (j) < last ? (j) : last;                                                  \
        const size_t off_ = static_cast<size_t>(j_) * kt_stride - ((2 * j_ + 1 >= g.KS && (tid & 7) >= 4) ? 64 : 0); \
        if (loader) {                                                                            \
            _Pragma("unroll") for (int q = 0; q < kLoadsB; ++q)                                  \
                breg[set][q] = *reinterpret_cast<const bf16x8 *>(bp[q] + off_);                  \
        }                                                                                        \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
#define MOE_WIDE_STAGE(set)                                                                      \
    do {                                                                                         \
        if (loader) {                                                                            \
            _Pragma("unroll") for (int q = 0; q < kLoadsB; ++q)                                  \
                *reinterpret_cast<bf16x8 *>(lds + ((set) & 1) * kBufBytes + q * (kThreads * 16) + wr_lds) = breg[set][q]; \
        }                                                                                        \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
    // the multiply of one K-step: row tiles in groups of up to four (LDS reads of a group, then its MFMAs)
#define MOE_WIDE_MMA_STEP(set, ss)                                                               \
    do {                                                                                         \
        _Pragma("unroll") for (int r0_ = 0; r0_ < RT; r0_ += 4) {                                \
            bf16x8 b_[4];                                                                        \
            _Pragma("unroll") for (int r4 = 0; r4 < 4; ++r4)                                     \
                if (r0_ + r4 < RT)                                                               \
                    b_[r4] = *reinterpret_cast<const bf16x8 *>(                                  \
                        lds + ((set) & 1) * kBufBytes + (r0_ + r4) * 2048 + rd_row + (((4 * (ss) + rd_g) ^ rd_sw) * 16)); \
            _Pragma("unroll") for (int r4 = 0; r4 < 4; ++r4)                                     \
                if (r0_ + r4 < RT) {                                                             \
                    acc[r0_ + r4][0] = mfma16(areg[set][ss][0], b_[r4], acc[r0_ + r4][0]);       \
                    acc[r0_ + r4][1] = mfma16(areg[set][ss][1], b_[r4], acc[r0_ + r4][1]);       \
                }                                                                                \
        }                                                                                        \
    } while (0)
    // The LDS buffer written here was last read in the multiply of K-tile i-2, which every wavefront
    // finished before the barrier of K-tile i-1.  full: both K-steps of the tile exist (a literal).
#define MOE_WIDE_STEP(set, i, full)                                                              \
    do {                                                                                         \
        MOE_WIDE_STAGE(set);                                                                     \
        MOE_WIDE_LOAD_B(set, (i) + kRing);                                                       \
        lds_barrier();                                                                           \
        MOE_WIDE_MMA_STEP(set, 0);                                                               \
        if (full) MOE_WIDE_MMA_STEP(set, 1);                                                     \
        asm volatile("" ::: "memory");                                                           \
        MOE_WIDE_LOAD_A(set, (i) + kRing);                                                       \
    } while (0)

    const int n_full = g.KS >> 1;                                    // K-tiles with both K-steps
    int i = 0;
    MOE_WIDE_LOAD_A(0, 0); MOE_WIDE_LOAD_B(0, 0);
    MOE_WIDE_LOAD_A(1, 1); MOE_WIDE_LOAD_B(1, 1);
    for (; i + 2 <= n_full; i += 2) {
        MOE_WIDE_STEP(0, i, true);
        MOE_WIDE_STEP(1, i + 1, true);
    }
    const int rem = n_full - i;                                      // 0 .. 1
    if (rem > 0) MOE_WIDE_STEP(0, i, true);
    if (g.KS & 1) {
        if (rem == 0) MOE_WIDE_STEP(0, n_full, false);
        else MOE_WIDE_STEP(1, n_full, false);
    }
#undef MOE_WIDE_LOAD_A
#undef MOE_WIDE_LOAD_B
#undef MOE_WIDE_STAGE
#undef MOE_WIDE_MMA_STEP
#undef MOE_WIDE_STEP

    // lane l holds, per row tile, 4 consecutive channels (l/16)*4.. of row (l%16) of the tile
    if (pt_ok) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const int r = rt * 16 + (lane & 15);
            if (r >= m) continue;
            if constexpr (STAGE1) {
                const f32x4 gt = acc[rt][0], up = acc[rt][1];
                const uint64_t o = static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(gt[0], up[0]))) |
                                   static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(gt[1], up[1]))) << 16 |
                                   static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(gt[2], up[2]))) << 32 |
                                   static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(gt[3], up[3]))) << 48;
                uint64_t *dst = reinterpret_cast<uint64_t *>(act_blk + (static_cast<size_t>(group) * rows_pad + r) * 128 +
                                                             wave * 32 + (lane >> 4) * 8);
                __hip_atomic_store(dst, o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                float *dst = a.Yp + static_cast<size_t>(row0 + r) * g.out_stride + pt * 32 + (lane >> 4) * 4;
                *reinterpret_cast<f32x4 *>(dst) = acc[rt][0];
                *reinterpret_cast<f32x4 *>(dst + 16) = acc[rt][1];
            }
        }
    }
    if constexpr (STAGE1) {
        // announce the tile group: stores acknowledged, then the counter of the leading entry
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            int *blk = a.ctrl + (item + 1) * kCtrlBlockInts;
            if (__hip_atomic_fetch_add(blk, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_groups - 1) {
#pragma unroll
                for (int c = 1; c <= kCtrlCopies; ++c)
                    __hip_atomic_store(blk + c * kCtrlLineInts, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// A slot with more than kWideMin requests is wide.  Its rows are cut into blocks of WR = 64 rows (a block
// of 128 rows needs 64 accumulator registers more than the streaming items leave at three workgroups
// per CU; batches of thousands of tokens take the tiled-GEMM launches of ffn_wide.hip instead).
constexpr int kWideMin = 64;
// A wavefront of a wide workgroup runs its tile's whole K dimension, one round trip per K-tile (about
// kWideTileNs each), so a wide workgroup lasts much longer than a streaming item.  Wide blocks pay off
//  - when a batch has enough of them to fill the chip with such workgroups: (64-row blocks of the wide
//    slots, from the list's header) x (first-stage workgroups per block) >= kWideMinWorkgroups; or
//  - from kWideMinHidden workgroups on, when the rest of the launch lasts long enough to hide them (they
//    come first in the list and start with the launch): the time the launch needs to stream one expert
//    per list entry at kStreamBytesPerNs must exceed 5/4 of the K-tiles of both stages x kWideTileNs.
// Otherwise the wide slots are cut into streaming items like the others.  Every workgroup takes the
// decision from the same numbers.  A caller's threshold replaces the first rule and switches the
// second off.
constexpr int kWideMinWorkgroups = 256;
constexpr int kWideMinHidden = 64;
constexpr long long kWideTileNs = 900, kStreamBytesPerNs = 7000;
__device__ __forceinline__ bool wide_on(int4 head, int groups1, int override_min, int ks1, int ks2) {
    const int wgs = head.z * groups1;
    if (override_min > 0) return wgs >= override_min;
    if (wgs >= kWideMinWorkgroups) return true;
    if (wgs < kWideMinHidden) return false;
    // an expert's three matrices: 3 * d_h * d_e bf16 = ks1 * ks2 * 32 * 32 * 6 bytes
    const long long stream_ns = static_cast<long long>(head.x) * ks1 * ks2 * (32 * 32 * 6) / kStreamBytesPerNs;
    const long long chain_ns = static_cast<long long>((ks1 + 1) / 2 + (ks2 + 1) / 2) * kWideTileNs;
    return 4 * stream_ns >= 5 * chain_ns;
}
// The workgroups of a wide slot's leading entries (one entry per block of WR rows; ids tile = 0 .. tiles_pad-1
// each) run the slot's blocks x groups of 4 tiles; all other workgroups of the slot's entries leave.
// Workgroup ids go round-robin over the eight XCDs, so tile % 8 is the XCD and (leader index, tile / 8)
// the place in that XCD's start order.  That order is walked block-fastest: the blocks of one group of
// tiles start next to each other on one XCD, walk the expert's tiles side by side, and all but the first
// find them in that L2.  (Group-fastest, the natural order of the ids, put the sibling blocks tiles_pad / 8
// starts apart: on a busy chip that is longer than a line survives in a streaming L2, and every block of a
// slot fetched the expert from memory again.)  BR = rows per list entry.
template <bool STAGE1, int WR, int BR>
__device__ __forceinline__ void run_wide(const StreamArgs &a, const StageArgs &g, char *lds, int *s_ok, int item,
                                         int tile, int4 ent) {
    const int slot = ent.x, hi = ent.z, lo = ent.w;
    if ((ent.y - lo) % WR != 0) return;                              // not the leading entry of a wide block
    const int groups = (g.tiles + kWaves - 1) / kWaves;              // workgroups of a block in this stage
    const int nb = (hi - lo + WR - 1) / WR;                          // blocks of the slot
    const int leader = (ent.y - lo) / WR;                            // which of them this entry leads
    const int xcd = tile & 7;
    const int place = leader * (g.tiles_pad >> 3) + (tile >> 3);     // in the XCD's start order, within the slot
    const int group = xcd + 8 * (place / nb), b = place % nb;
    if (group >= groups) return;
    item += (b - leader) * (WR / BR);                                // the block's leading entry: its control lines and `act`
    const int row0 = lo + b * WR;
    const int m = hi - row0 < WR ? hi - row0 : WR;
    const int rt = (m + 15) >> 4;
    if (rt <= 1) wide_item<STAGE1, 1>(a, g, lds, s_ok, item, group, groups, slot, row0, m);
    else if (rt <= 2) wide_item<STAGE1, 2>(a, g, lds, s_ok, item, group, groups, slot, row0, m);
    else wide_item<STAGE1, 4>(a, g, lds, s_ok, item, group, groups, slot, row0, m);
}

// LINES: this stage has an even number of K-steps
// wide: 0 = every slot is cut into streaming items; 1 = slots with more than kWideMin requests are wide
// blocks of this launch; 2 = those slots belong to the tiled-GEMM launches and are skipped here
template <bool STAGE1, bool LINES, int TT, int WR>
__device__ __forceinline__ void run_item(const StreamArgs &a, const StageArgs &g, char *lds, int *s_ok, int wide,
                                         unsigned id) {
    int tile = id % g.tiles_pad;
    const int item = id / g.tiles_pad;
    // work list entry: {slot, first row, end of the slot's rows, first of the slot's rows}; entry 0 holds the number of blocks
    // (both are wave-uniform scalar loads issued together; an entry past the end is never used)
    const int4 *list = reinterpret_cast<const int4 *>(a.blocks);
    const int n_blocks = list[0].x;
    const int4 ent = list[1 + item];
    if (item >= n_blocks) return;                                // past the last block: nothing else is read
    // a slot with more than kWideRows requests is computed as tiled GEMMs over blocks of kWideRows rows
    if (wide && ent.z - ent.w > kWideMin) {
        if (wide == 1) run_wide<STAGE1, WR, TT * 16>(a, g, lds, s_ok, item, tile, ent);
        return;
    }
    if (tile >= g.items) return;                                 // ids that pad the tiles to a multiple of 8
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE), lane = threadIdx.x % MOE_WAVE;
    const int slot = ent.x, row0 = ent.y, hi = ent.z;
    // in the 64-row launch a stage-2 workgroup owns a pair of tiles (larger batches: the pairs halve
    // the workgroup turnover of the second stage; small batches want every tile on a workgroup of its own)
    constexpr bool kPairs = !STAGE1 && TT == 4;
    if constexpr (kPairs) tile *= 2;
    const char *w = g.Wp + (static_cast<size_t>(slot) * g.tiles + tile) * g.KS * 2048;
    const int m = hi - row0;
    const bool single = m <= TT * 16 && row0 == ent.w;                  // the slot's only block
    if constexpr (!STAGE1) {
        const int tiles16 = ((m < TT * 16 ? m : TT * 16) + 15) >> 4;     // 16-row token tiles that hold requests
        const bool two = kPairs && tile + 1 < g.tiles;                   // an odd number of tiles leaves the last one alone
        // blocks with few rows multiply both tiles at once (every workgroup of a block takes the same
        // branch, so the block's readers are counted the same way by all)
        const bool paired = kPairs && tiles16 <= 2;
#define MOE_DOWN(NT, U, NW, t_, n_readers_)                                                          \
        do {                                                                                         \
            const char *w_ = w + static_cast<size_t>((t_) - tile) * g.KS * 2048;                     \
            if (single) stream_item_down<NT, TT, U, true, NW>(a, g, lds, s_ok, w_, item, t_, n_readers_, row0, hi, wave, lane);  \
            else stream_item_down<NT, TT, U, false, NW>(a, g, lds, s_ok, w_, item, t_, n_readers_, row0, hi, wave, lane);        \
        } while (0)
#define MOE_CASE_PAIR(NT, U)                                                                         \
    case NT:                                                                                         \
        if (two) MOE_DOWN(NT, U, 2, tile, g.items);                                                  \
        else MOE_DOWN(NT, U, 1, tile, g.items);                                                      \
        break;
#define MOE_CASE_SEQ(NT, U)                                                                          \
    case NT:                                                                                         \
        MOE_DOWN(NT, U, 1, tile, g.tiles);                                                           \
        if (two) {                                                                                   \
            __syncthreads();                                             /* the LDS buffer is reused */ \
            MOE_DOWN(NT, U, 1, tile + 1, g.tiles);                                                   \
        }                                                                                            \
        break;
        if constexpr (TT == 2) {
            switch (tiles16) { MOE_CASE_SEQ(1, LINES ? 2 : 1) MOE_CASE_SEQ(2, LINES ? 2 : 1) }
        } else if (paired) {
            switch (tiles16) { MOE_CASE_PAIR(1, LINES ? 2 : 1) MOE_CASE_PAIR(2, LINES ? 2 : 1) }
        } else {
            switch (tiles16) { MOE_CASE_SEQ(3, 1) MOE_CASE_SEQ(4, 1) }
        }
#undef MOE_DOWN
#undef MOE_CASE_PAIR
#undef MOE_CASE_SEQ
    } else if (LINES) {
        const int halves = ((m < TT * 16 ? m : TT * 16) + 7) >> 3;     // 8-row halves that hold requests
#define MOE_CASE(NH)                                                                                 \
    case NH:                                                                                         \
        if (single) stream_item_lines<NH, TT, true>(a, g, lds, w, item, tile, row0, hi, wave, lane);    \
        else stream_item_lines<NH, TT, false>(a, g, lds, w, item, tile, row0, hi, wave, lane);          \
        break;
        if constexpr (TT == 2) {
            switch (halves) { MOE_CASE(1) MOE_CASE(2) MOE_CASE(3) MOE_CASE(4) }
        } else {
            switch (halves) { MOE_CASE(1) MOE_CASE(2) MOE_CASE(3) MOE_CASE(4) MOE_CASE(5) MOE_CASE(6) MOE_CASE(7) MOE_CASE(8) }
        }
#undef MOE_CASE
    } else {
        // passes of 32 rows (rows [row0 + brow, ...) of the block)
        const int end = m < TT * 16 ? hi : row0 + TT * 16;
        for (int brow = 0; row0 + brow < end; brow += 32) {
            if (brow) __syncthreads();                           // the reduction buffer is reused
            if (end - (row0 + brow) <= 16) stream_item_steps<1, TT>(a, g, lds, w, item, brow, tile, row0 + brow, end, wave, lane);
            else stream_item_steps<2, TT>(a, g, lds, w, item, brow, tile, row0 + brow, end, wave, lane);
        }
    }
    if (STAGE1) {
        // announce the tile: every thread waits for its own act stores to be acknowledged, then
        // one thread bumps the block's counter and, if it completes the count, raises the ready flags
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0) {
            int *blk = a.ctrl + (item + 1) * kCtrlBlockInts;
            if (__hip_atomic_fetch_add(blk, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == g.tiles - 1) {
                // last tile of the block: every other tile's stores were acknowledged before its bump
#pragma unroll
                for (int c = 1; c <= kCtrlCopies; ++c)
                    __hip_atomic_store(blk + c * kCtrlLineInts, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// 1-D grid sized for the worst case (at most kFfnLaneBlocks blocks).  With B = min(the batch's number of
// blocks, kFfnLaneBlocks), ids below B*tiles_pad(1) are the stage-1 workgroups (id = block * tiles_pad +
// tile), the next B*tiles_pad(2) ids the stage-2 workgroups, and the rest leave at once.  Workgroups are dispatched in id order, so a
// stage-2 workgroup is started after every stage-1 workgroup, and go to the XCDs round-robin, so
// the blocks of one tile of a slot (ids tiles_pad apart, a multiple of 8) run on the same XCD at
// about the same time: the tile's weights come from HBM once and are shared through that XCD's
// L2.  LINES1 / LINES2 select the whole-line token path of a stage (even number of K-steps).
// TT = token tiles per block (2: blocks of 32 rows, 4 workgroups per CU; 4: blocks of 64 rows, whose
// larger register set allows 3 per CU).
template <bool LINES1, bool LINES2, int TT, int WR>
__global__ __launch_bounds__(kThreads, TT == 2 ? 4 : 3)
void ffn_stream_kernel(StreamArgs a) {
    // split-K reduction buffer [4 waves][2][TT][64] x 16 B, which the whole-line path also uses as
    // its per-wavefront staging tiles during the K loop
    __shared__ __attribute__((aligned(16))) char lds[kWaves * 2 * TT * MOE_WAVE * 16];
    static_assert(kWaves * TT * 2048 <= sizeof(lds), "staging tiles must fit in the reduction buffer");
    static_assert(2 * WR * 128 <= sizeof(lds), "the two token tiles of a wide block must fit");
    __shared__ unsigned long long s_visit;
    __shared__ int s_ok;
    {
        // ids are decoded with the number of blocks the batch really has, so that the surplus of
        // the worst-case grid comes after all the work of both stages
        const int4 head = reinterpret_cast<const int4 *>(a.blocks)[0];
        if (head.y != TT * 16) {
            // the list was cut for another block size (made for a different T): refuse, visibly
            if (threadIdx.x == 0 && blockIdx.x == 0)
                __hip_atomic_fetch_or(a.ctrl + moe::kCtrlStatus, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }

        // Up to kFfnLaneBlocks blocks have workgroups of their own; a longer list wraps around (the
        // workgroup of block b also takes blocks b + kFfnLaneBlocks, ..., at most 64 of them), which
        // keeps the worst-case grid of large batches small.  A stage-1 workgroup never waits, and all of them are started
        // before any stage-2 workgroup, so every flag a stage-2 workgroup waits for is raised.
        // header word 3 of the workspace: the caller's threshold for wide blocks (0 = default)
        const int wide_min = a.ctrl[moe::kCtrlWideMin];
        const int wide = a.has_gemm && moe::ffn_gemm_on(head, (a.s[0].tiles + kWaves - 1) / kWaves, wide_min) ? 2
                         : wide_on(head, (a.s[0].tiles + kWaves - 1) / kWaves, wide_min, a.s[0].KS, a.s[1].KS) ? 1 : 0;
        const unsigned n_blocks = static_cast<unsigned>(head.x);
        const unsigned lanes = n_blocks < moe::kFfnLaneBlocks ? n_blocks : moe::kFfnLaneBlocks;
        const unsigned n1 = lanes * a.s[0].tiles_pad, n2 = lanes * a.s[1].tiles_pad;
        if (n_blocks <= lanes) {
            if (blockIdx.x < n1) run_item<true, LINES1, TT, WR>(a, a.s[0], lds, &s_ok, wide, blockIdx.x);
            else if (blockIdx.x - n1 < n2) run_item<false, LINES2, TT, WR>(a, a.s[1], lds, &s_ok, wide, blockIdx.x - n1);
        } else if (blockIdx.x < n1 + n2) {
            // a long list: the first wavefront looks at all the blocks of this workgroup at once (lane l:
            // block + l*lanes) and the workgroup then visits only those that are its own to compute
            const bool s1 = blockIdx.x < n1;
            const unsigned id0 = s1 ? blockIdx.x : blockIdx.x - n1;
            const unsigned tp = s1 ? a.s[0].tiles_pad : a.s[1].tiles_pad;
            // (ids that pad the tiles to a multiple of 8 stay: the wide slots use them)
            if (threadIdx.x < MOE_WAVE) {
                const unsigned b = id0 / tp + threadIdx.x * lanes;
                // entries of wide slots that lead no block are not visited
                bool mine = false;
                if (b < n_blocks) {
                    const int4 e = reinterpret_cast<const int4 *>(a.blocks)[1 + b];
                    mine = !wide || e.z - e.w <= kWideMin || (wide == 1 && (e.y - e.w) % WR == 0);
                }
                const unsigned long long m = __ballot(mine);
                if (threadIdx.x == 0) s_visit = m;
            }
            __syncthreads();
            unsigned long long visit = s_visit;
            bool first = true;
            while (visit) {
                const unsigned l = static_cast<unsigned>(__builtin_ctzll(visit));
                visit &= visit - 1;
                if (!first) __syncthreads();                         // the LDS buffer is reused
                first = false;
                if (s1) run_item<true, LINES1, TT, WR>(a, a.s[0], lds, &s_ok, wide, id0 + l * n1);
                else run_item<false, LINES2, TT, WR>(a, a.s[1], lds, &s_ok, wide, id0 + l * n2);
            }
        }
    }
}

template <bool L1, bool L2>
void launch(const StreamArgs &a, int block_rows, unsigned blocks, hipStream_t st) {
    if (block_rows == 32) hipLaunchKernelGGL((ffn_stream_kernel<L1, L2, 2, 64>), dim3(blocks), dim3(kThreads), 0, st, a);
    else hipLaunchKernelGGL((ffn_stream_kernel<L1, L2, 4, 64>), dim3(blocks), dim3(kThreads), 0, st, a);
}

void launch_lines(const StreamArgs &a, int block_rows, unsigned blocks, hipStream_t st) {
    const bool l1 = a.s[0].KS % 2 == 0, l2 = a.s[1].KS % 2 == 0;
    if (l1 && l2) launch<true, true>(a, block_rows, blocks, st);
    else if (l1) launch<true, false>(a, block_rows, blocks, st);
    else if (l2) launch<false, true>(a, block_rows, blocks, st);
    else launch<false, false>(a, block_rows, blocks, st);
}

}  // namespace

namespace moe {

int launch_ffn_stream(const void *X, const void *W13p, const void *W2p, int T, int k, int C, int d_h, int d_e,
                      const int32_t *blocks, const int32_t *perm, int *ctrl, uint16_t *act,
                      float *Yp, hipStream_t st) {
    const int block_rows = ffn_block_rows(T);
    const long long items = ffn_max_blocks(T, k, C);
    if (items > kMaxItems) return MOE_ESHAPE;
    StreamArgs a;
    a.blocks = blocks; a.perm = perm; a.act = act; a.Yp = Yp; a.ctrl = ctrl; a.k = k; a.C = C;
    a.spin_limit = 1 << 20;
    a.act_block_bytes = static_cast<uint32_t>(ffn_act_block_bytes(T, d_e));
    a.has_gemm = ffn_has_gemm(T) ? 1 : 0;
    a.s[0].B = static_cast<const uint16_t *>(X);
    a.s[0].Wp = static_cast<const char *>(W13p);
    a.s[0].tiles = d_e / 16; a.s[0].KS = d_h / 32; a.s[0].b_stride = d_h; a.s[0].out_stride = 0;
    a.s[1].B = act;
    a.s[1].Wp = static_cast<const char *>(W2p);
    a.s[1].tiles = d_h / 32; a.s[1].KS = d_e / 32; a.s[1].b_stride = 0; a.s[1].out_stride = d_h;
    a.s[0].items = a.s[0].tiles;
    a.s[1].items = block_rows == 32 ? a.s[1].tiles : (a.s[1].tiles + 1) / 2;   // 64-row launch: a stage-2 workgroup owns a pair of tiles
    for (int i = 0; i < 2; ++i) a.s[i].tiles_pad = (a.s[i].items + 7) / 8 * 8;
    const long long lanes = items < kFfnLaneBlocks ? items : kFfnLaneBlocks;
    const long long n1 = lanes * a.s[0].tiles_pad, n2 = lanes * a.s[1].tiles_pad;
    if (n1 + n2 > 0x7fffffffLL) return MOE_ESHAPE;
    launch_lines(a, block_rows, static_cast<unsigned>(n1 + n2), st);
    return MOE_OK;
}

}  // namespace moe

