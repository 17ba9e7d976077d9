// a5, bf16 path: the grouped expert FFN as two streaming launches (gate/up + SiLU*up, then down).
//
// Janus Sec. 2.2: at decode sizes an expert is two skinny GEMMs whose cost is the weight bytes
// streamed from HBM, so the layer's latency follows the number of activated experts.  The
// kernels below are plain oversubscribed streamers: one workgroup per (slot, 16- or 32-channel
// tile of the output) and K-split part, dispatched by the hardware; a workgroup of a slot
// without requests leaves at once and never touches that slot's weights.
//
// The 4 wavefronts of a workgroup split the K-steps (32 columns each) of the tile round-robin,
// keep kDepth steps of 128-bit loads in flight each (weights: 1 KiB MFMA A-operand images,
// fully coalesced; tokens: B operand fetched from L2), and meet in LDS once per pass of 32
// tokens.  The sum over wavefronts is taken in a fixed order, so results are reproducible.
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kDepth = 4;               // K-steps of loads each wavefront keeps in flight
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / MOE_WAVE;
constexpr int kMaxTiles = 2;            // token tiles (of 16) per workgroup
constexpr int kBlockTok = kMaxTiles * 16; // tokens of a slot one workgroup takes

#ifdef MOE_STREAM_TRACE
// timeline of every workgroup (debug builds only): [stage][linear id][start, first data, end, xcc/cu]
__device__ long long g_trace[2][1 << 15][4];
#endif

struct StreamArgs {
    const uint16_t *B;                   // token operand rows: X (stage 1, through perm) or act (stage 2)
    const bf16x8 *Wp;                    // packed weights: [C][tiles][KS][2][64] fragments
    const int32_t *slot_off;
    const int32_t *perm;
    uint16_t *act;                       // stage-1 output
    float *Yp;                           // stage-2 output
    int k, C, tiles, KS;
    int tiles_pad;                       // tiles rounded up to a multiple of 8
    int b_stride;                        // elements between rows of B
    int out_stride;                      // elements between rows of the output
};

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + __expf(-g)) * u; }

// Split-K reduction over the 4 wavefronts in LDS (fixed order), then the epilogue: SiLU(gate)*up
// rounded once to bf16 (stage 1) or the fp32 partial output rows (stage 2).
template <bool STAGE1, int NT>
__device__ __forceinline__ void reduce_store(const StreamArgs &a, f32x4 (*red)[2][kMaxTiles][MOE_WAVE],
                                             f32x4 (&acc)[2][NT], int tile, int row0, int row_end,
                                             int wave, int lane) {
    // split-K reduction over the 4 wavefronts in LDS, fixed order
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int t = 0; t < NT; ++t) red[wave][h][t][lane] = acc[h][t];
    __syncthreads();
    if (STAGE1) {
        // lane-slot (t, l) holds gate/up channels tile*16 + (l/16)*4 .. +3 of token row0 + t*16 + l%16
        for (int item = threadIdx.x; item < NT * MOE_WAVE; item += kThreads) {
            const int t = item / MOE_WAVE, l = item % MOE_WAVE;
            f32x4 g = red[0][0][t][l], u = red[0][1][t][l];
#pragma unroll
            for (int wv = 1; wv < kWaves; ++wv) { g += red[wv][0][t][l]; u += red[wv][1][t][l]; }
            const int r = row0 + t * 16 + (l & 15);
            if (r < row_end) {
                ushort4 o;
                o.x = moe::f32_to_bf16(silu_mul(g[0], u[0]));
                o.y = moe::f32_to_bf16(silu_mul(g[1], u[1]));
                o.z = moe::f32_to_bf16(silu_mul(g[2], u[2]));
                o.w = moe::f32_to_bf16(silu_mul(g[3], u[3]));
                *reinterpret_cast<ushort4 *>(a.act + static_cast<size_t>(r) * a.out_stride + tile * 16 + (l >> 4) * 4) = o;
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
                *reinterpret_cast<f32x4 *>(a.Yp + static_cast<size_t>(r) * a.out_stride + tile * 32 + h * 16 + (l >> 4) * 4) = y;
        }
    }
}

// One pass: tokens [row0, row0 + NT*16) of the slot (rows >= row_end are padding) against the
// workgroup's tile.  `w` points at K-step 0 of the tile (wave-uniform).  A wavefront advances in
// super-steps of SS consecutive K-steps (SS*2 KiB of weights, SS*64 contiguous bytes of every
// token row: SS = 2 reads whole 128-byte lines of the token rows) and keeps D super-steps in flight.
template <bool STAGE1, int NT, int SS>
__device__ __forceinline__ void stream_pass(const StreamArgs &a, f32x4 (*red)[2][kMaxTiles][MOE_WAVE],
                                            const char *w, int tile, int row0, int row_end,
                                            int wave, int lane) {
    constexpr int D = kDepth / SS;
    // B operand: lane l reads 8 columns (l/16)*8.. of token row l%16 of every token tile.  Weights
    // and tokens are both addressed as a wave-uniform base (scalar registers, advanced per K-step)
    // plus a constant 32-bit per-lane byte offset.
    const uint32_t aoff = lane * 16;
    uint32_t boff[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int r = row0 + t * 16 + (lane & 15);
        r = r < row_end ? r : row_end - 1;
        const uint32_t src = STAGE1 ? static_cast<uint32_t>(a.perm[r] / a.k) : static_cast<uint32_t>(r);
        boff[t] = (src * static_cast<uint32_t>(a.b_stride) + (lane >> 4) * 8) * 2;
    }
    const char *bbase = reinterpret_cast<const char *>(a.B);
    const int n = (a.KS / SS - wave + kWaves - 1) / kWaves;     // super-steps wave, wave+4, ... of this wavefront
    f32x4 acc[2][NT];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[h][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (n > 0) {
        // Ring entry d holds super-step i+d.  The steady-state loop has no branch, so the compiler
        // counts outstanding loads exactly and each MFMA waits only for its own entry.  Loads past
        // the last super-step fetch the last one again (a cache hit): every load is unconditional.
        bf16x8 wr[D][SS][2], br[D][SS][NT];
        const int last = n - 1;
        // Workgroups start their K loop at different places (and wrap around) so that they do not
        // march through equally aligned tiles in lockstep.
        const int rot = static_cast<int>(static_cast<unsigned>(tile) % static_cast<unsigned>(n));
#define MOE_LOAD_STEP(d, step)                                                                   \
        do {                                                                                     \
            const int q_ = (step);                                                               \
            int r_ = (q_ < last ? q_ : last) + rot;                                              \
            r_ = r_ >= n ? r_ - n : r_;                                                          \
            const int s_ = wave + kWaves * r_;                                                   \
            const char *ws_ = w + static_cast<size_t>(s_) * (2048 * SS);                         \
            const char *bs_ = bbase + static_cast<size_t>(s_) * (64 * SS);                       \
            _Pragma("unroll") for (int ss = 0; ss < SS; ++ss) {                                  \
                wr[d][ss][0] = *reinterpret_cast<const bf16x8 *>(ws_ + ss * 2048 + aoff);        \
                wr[d][ss][1] = *reinterpret_cast<const bf16x8 *>(ws_ + ss * 2048 + 1024 + aoff); \
            }                                                                                    \
            _Pragma("unroll") for (int t = 0; t < NT; ++t)                                       \
                _Pragma("unroll") for (int ss = 0; ss < SS; ++ss)                                \
                    br[d][ss][t] = *reinterpret_cast<const bf16x8 *>(bs_ + ss * 64 + boff[t]);   \
            asm volatile("" ::: "memory");                                                       \
        } while (0)
#define MOE_MMA_STEP(d)                                                                          \
        do {                                                                                     \
            _Pragma("unroll") for (int ss = 0; ss < SS; ++ss)                                    \
                _Pragma("unroll") for (int t = 0; t < NT; ++t) {                                 \
                    acc[0][t] = mfma16(wr[d][ss][0], br[d][ss][t], acc[0][t]);                   \
                    acc[1][t] = mfma16(wr[d][ss][1], br[d][ss][t], acc[1][t]);                   \
                }                                                                                \
        } while (0)
#pragma unroll
        for (int d = 0; d < D; ++d) MOE_LOAD_STEP(d, d);
        int i = 0;
        for (; i + 2 * D <= n; i += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                MOE_MMA_STEP(d);
                MOE_LOAD_STEP(d, i + d + D);
            }
        }
        const int rem = n - i;                                   // 1 .. 2*D-1 super-steps left
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (d < rem) MOE_MMA_STEP(d);
            if (d < D - 1) MOE_LOAD_STEP(d, i + d + D);
        }
#pragma unroll
        for (int d = 0; d < D - 1; ++d)
            if (D + d < rem) MOE_MMA_STEP(d);
#undef MOE_LOAD_STEP
#undef MOE_MMA_STEP
    }

    reduce_store<STAGE1, NT>(a, red, acc, tile, row0, row_end, wave, lane);
}

// The same pass for an even number of K-steps, with whole-line token reads.  A super-step is two
// K-steps = 64 columns = one 128-byte line of every token row.  A load instruction fetches 8 rows
// x 128 bytes (lane l: row l/8, 16-byte chunk l%8), so no line is requested twice and none by
// halves; the MFMA layout (lane l: row l%16, chunk 4*step + l/16) is produced by a round trip
// through a wave-private 2 KiB LDS tile per 16 rows (chunks XOR-swizzled by row so that both the
// row-major writes and the column-wise reads spread over the banks).  NH = number of 8-row halves
// that hold requests (rows past the end repeat the last row; halves past it are not loaded and
// leave unspecified values in token columns whose results are never stored).
template <bool STAGE1, int NH>
__device__ __forceinline__ void stream_pass_lines(const StreamArgs &a, char *lds, const char *w, int tile,
                                                  int row0, int row_end, int wave, int lane) {
    constexpr int NT = (NH + 1) / 2;
    constexpr int D = kDepth / 2;
    f32x4 (*red)[2][kMaxTiles][MOE_WAVE] = reinterpret_cast<f32x4 (*)[2][kMaxTiles][MOE_WAVE]>(lds);
    char *stg = lds + wave * (kMaxTiles * 2048);
    const uint32_t aoff = lane * 16;
    uint32_t boff[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        int r = row0 + h * 8 + (lane >> 3);
        r = r < row_end ? r : row_end - 1;
        const uint32_t src = STAGE1 ? static_cast<uint32_t>(a.perm[r] / a.k) : static_cast<uint32_t>(r);
        boff[h] = src * static_cast<uint32_t>(a.b_stride) * 2 + (lane & 7) * 16;
    }
    // LDS addresses: write row (h%2)*8 + l/8 of tile h/2, chunk l%8; read row l%16, chunk 4*ss + l/16
    const uint32_t wr_lds = ((lane >> 3) * 128) + (((lane & 7) ^ (lane >> 3)) * 16);
    const uint32_t rd_row = (lane & 15) * 128, rd_sw = lane & 7, rd_g = lane >> 4;
    const char *bbase = reinterpret_cast<const char *>(a.B);
    const int n = (a.KS / 2 - wave + kWaves - 1) / kWaves;      // super-steps wave, wave+4, ... of this wavefront
    f32x4 acc[2][NT];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[h][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (n > 0) {
        // Weights run D super-steps ahead (ring wr); the token rows, which come from L2, only one:
        // the loads of super-step q+1 are issued in iteration q *before* the weights of q+D, so that
        // waiting for them (loads return in order) leaves those weights in flight.
        bf16x8 wr[D][2][2], br[NH];
        const int last = n - 1;
        const int rot = static_cast<int>(static_cast<unsigned>(tile) % static_cast<unsigned>(n));
#define MOE_STEP_INDEX(step)                                                                     \
            const int q_ = (step);                                                               \
            int r_ = (q_ < last ? q_ : last) + rot;                                              \
            r_ = r_ >= n ? r_ - n : r_;                                                          \
            const int s_ = wave + kWaves * r_;
#define MOE_LOAD_A(d, step)                                                                      \
        do {                                                                                     \
            MOE_STEP_INDEX(step)                                                                 \
            const char *ws_ = w + static_cast<size_t>(s_) * 4096;                                \
            _Pragma("unroll") for (int ss = 0; ss < 2; ++ss) {                                   \
                wr[d][ss][0] = *reinterpret_cast<const bf16x8 *>(ws_ + ss * 2048 + aoff);        \
                wr[d][ss][1] = *reinterpret_cast<const bf16x8 *>(ws_ + ss * 2048 + 1024 + aoff); \
            }                                                                                    \
            asm volatile("" ::: "memory");                                                       \
        } while (0)
#define MOE_LOAD_B(step)                                                                         \
        do {                                                                                     \
            MOE_STEP_INDEX(step)                                                                 \
            const char *bs_ = bbase + static_cast<size_t>(s_) * 128;                             \
            _Pragma("unroll") for (int h = 0; h < NH; ++h)                                       \
                br[h] = *reinterpret_cast<const bf16x8 *>(bs_ + boff[h]);                        \
            asm volatile("" ::: "memory");                                                       \
        } while (0)
#define MOE_STAGE_B()                                                                            \
        do {                                                                                     \
            _Pragma("unroll") for (int h = 0; h < NH; ++h)                                       \
                *reinterpret_cast<bf16x8 *>(stg + (h / 2) * 2048 + (h % 2) * 1024 + wr_lds) = br[h]; \
            asm volatile("" ::: "memory");                                                       \
        } while (0)
#define MOE_MMA_STEP(d)                                                                          \
        do {                                                                                     \
            _Pragma("unroll") for (int ss = 0; ss < 2; ++ss)                                     \
                _Pragma("unroll") for (int t = 0; t < NT; ++t) {                                 \
                    const bf16x8 bf_ = *reinterpret_cast<const bf16x8 *>(                        \
                        stg + t * 2048 + rd_row + (((4 * ss + rd_g) ^ rd_sw) * 16));             \
                    acc[0][t] = mfma16(wr[d][ss][0], bf_, acc[0][t]);                            \
                    acc[1][t] = mfma16(wr[d][ss][1], bf_, acc[1][t]);                            \
                }                                                                                \
            asm volatile("" ::: "memory");                                                       \
        } while (0)
        MOE_LOAD_B(0);
#pragma unroll
        for (int d = 0; d < D; ++d) MOE_LOAD_A(d, d);
        int i = 0;
        for (; i + 2 * D <= n; i += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                MOE_STAGE_B();
                MOE_LOAD_B(i + d + 1);
                MOE_MMA_STEP(d);
                MOE_LOAD_A(d, i + d + D);
            }
        }
        const int rem = n - i;                                   // 1 .. 2*D-1 super-steps left
#pragma unroll
        for (int d = 0; d < D; ++d) {
            MOE_STAGE_B();
            MOE_LOAD_B(i + d + 1);
            if (d < rem) MOE_MMA_STEP(d);
            if (d < D - 1) MOE_LOAD_A(d, i + d + D);
        }
#pragma unroll
        for (int d = 0; d < D - 1; ++d) {
            MOE_STAGE_B();
            if (d < D - 2) MOE_LOAD_B(i + D + d + 1);
            if (D + d < rem) MOE_MMA_STEP(d);
        }
#undef MOE_STEP_INDEX
#undef MOE_LOAD_A
#undef MOE_LOAD_B
#undef MOE_STAGE_B
#undef MOE_MMA_STEP
    }
    __syncthreads();                                             // the staging tiles are reused for the reduction
    reduce_store<STAGE1, NT>(a, red, acc, tile, row0, row_end, wave, lane);
}

__device__ __forceinline__ int wave_scan_inclusive(int v, int lane) {
#pragma unroll
    for (int off = 1; off < MOE_WAVE; off <<= 1) {
        const int o = __shfl_up(v, off, MOE_WAVE);
        if (lane >= off) v += o;
    }
    return v;
}

// Work item j of the launch: the j-th block of kBlockTok tokens when the blocks of all slots are
// listed in slot order (blocks of a slot adjacent).  Every wavefront works this out for itself
// from slot_off (C <= 256 slots, 4 per lane).  Returns false past the last block.
__device__ __forceinline__ bool find_item(const int32_t *__restrict__ slot_off, int C, int j, int lane,
                                          int *slot, int *blk) {
    int base = 0;
    for (int c0 = 0; c0 < C; c0 += MOE_WAVE) {
        const int sidx = c0 + lane;
        const int cnt = sidx < C ? slot_off[sidx + 1] - slot_off[sidx] : 0;
        const int v = (cnt + kBlockTok - 1) / kBlockTok;
        const int incl = wave_scan_inclusive(v, lane);
        const int lo = base + incl - v;
        const uint64_t hit = __ballot(v > 0 && j >= lo && j < lo + v);
        if (hit) {
            const int l = __builtin_ctzll(hit);
            *slot = c0 + l;
            *blk = j - __builtin_amdgcn_readlane(lo, l);
            return true;
        }
        base += __builtin_amdgcn_readlane(incl, MOE_WAVE - 1);
    }
    return false;
}

// 1-D grid: workgroup id = item * tiles_pad + tile (tiles_pad = tiles rounded up to a multiple of
// 8).  Workgroups are dispatched in id order and go to the XCDs round-robin, so the token blocks
// of one tile of a slot (ids tiles_pad apart) run on the same XCD at about the same time: the
// tile's weights come from HBM once and are shared through that XCD's L2.  LINES selects the
// whole-line token path (even number of K-steps).
template <bool STAGE1, bool LINES>
__global__ __launch_bounds__(kThreads, 4)
void ffn_stream_kernel(StreamArgs a) {
    // split-K reduction buffer [4 waves][2][kMaxTiles][64] x 16 B, which the whole-line path also
    // uses as its per-wavefront staging tiles during the K loop
    __shared__ __attribute__((aligned(16))) char lds[kWaves * 2 * kMaxTiles * MOE_WAVE * 16];
    static_assert(kWaves * kMaxTiles * 2048 <= sizeof(lds), "staging tiles must fit in the reduction buffer");
#ifdef MOE_STREAM_TRACE
    const long long t_start = wall_clock64();
    const unsigned lin = blockIdx.x;
#endif
    const int tile = blockIdx.x % a.tiles_pad, item = blockIdx.x / a.tiles_pad;
    if (tile >= a.tiles) return;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE), lane = threadIdx.x % MOE_WAVE;
    int slot, blk;
    if (!find_item(a.slot_off, a.C, item, lane, &slot, &blk)) return;   // past the last block: nothing is read
    const int lo = a.slot_off[slot], hi = a.slot_off[slot + 1];
    const int row0 = lo + blk * kBlockTok;
    const char *w = reinterpret_cast<const char *>(a.Wp) + (static_cast<size_t>(slot) * a.tiles + tile) * a.KS * 2048;
    const int m = hi - row0;
    if (LINES) {
        if (m <= 8) stream_pass_lines<STAGE1, 1>(a, lds, w, tile, row0, hi, wave, lane);
        else if (m <= 16) stream_pass_lines<STAGE1, 2>(a, lds, w, tile, row0, hi, wave, lane);
        else if (m <= 24) stream_pass_lines<STAGE1, 3>(a, lds, w, tile, row0, hi, wave, lane);
        else stream_pass_lines<STAGE1, 4>(a, lds, w, tile, row0, hi, wave, lane);
    } else {
        // odd number of K-steps: half-line token reads
        f32x4 (*red)[2][kMaxTiles][MOE_WAVE] = reinterpret_cast<f32x4 (*)[2][kMaxTiles][MOE_WAVE]>(lds);
        if (m <= 16) stream_pass<STAGE1, 1, 1>(a, red, w, tile, row0, hi, wave, lane);
        else stream_pass<STAGE1, 2, 1>(a, red, w, tile, row0, hi, wave, lane);
    }
#ifdef MOE_STREAM_TRACE
    if (threadIdx.x == 0 && lin < (1u << 15)) {
        unsigned hwid;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(hwid));
        unsigned hw2;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw2));
        long long *tr = g_trace[STAGE1 ? 0 : 1][lin];
        tr[0] = t_start; tr[1] = hi - row0; tr[2] = wall_clock64(); tr[3] = (static_cast<long long>(hwid) << 32) | hw2;
    }
#endif
}

// A slot receives at most one request per token (a token's k experts are distinct), so the
// launch has at most min(C * ceil(T/kBlockTok), C + T*k/kBlockTok) token blocks.
template <bool STAGE1>
void launch_stage(StreamArgs &a, int T, hipStream_t st) {
    const long long per_slot = (T + kBlockTok - 1) / kBlockTok;
    long long items = a.C * per_slot;
    const long long by_rows = a.C + static_cast<long long>(T) * a.k / kBlockTok;
    if (by_rows < items) items = by_rows;
    a.tiles_pad = (a.tiles + 7) / 8 * 8;
    const dim3 grid(static_cast<unsigned>(items * a.tiles_pad));
    if (a.KS % 2 == 0) hipLaunchKernelGGL((ffn_stream_kernel<STAGE1, true>), grid, dim3(kThreads), 0, st, a);
    else hipLaunchKernelGGL((ffn_stream_kernel<STAGE1, false>), grid, dim3(kThreads), 0, st, a);
}

}  // namespace

namespace moe {

// Launches both stages on `st`.  Shapes were validated by the caller (d_h, d_e multiples of 32).
void launch_ffn_stream(const void *X, const void *W13p, const void *W2p, int T, int k, int C, int d_h, int d_e,
                       const int32_t *slot_off, const int32_t *perm, uint16_t *act, int act_stride,
                       float *Yp, hipStream_t st) {
    // a slot receives at most one request per token, so T bounds its rows
    StreamArgs a;
    a.slot_off = slot_off; a.perm = perm; a.act = act; a.Yp = Yp; a.k = k; a.C = C;
    a.B = static_cast<const uint16_t *>(X);
    a.Wp = static_cast<const bf16x8 *>(W13p);
    a.tiles = d_e / 16; a.KS = d_h / 32; a.b_stride = d_h; a.out_stride = act_stride;
    launch_stage<true>(a, T, st);
    a.B = act;
    a.Wp = static_cast<const bf16x8 *>(W2p);
    a.tiles = d_h / 32; a.KS = d_e / 32; a.b_stride = act_stride; a.out_stride = d_h;
    launch_stage<false>(a, T, st);
}

}  // namespace moe

#ifdef MOE_STREAM_TRACE
extern "C" int moe_debug_stream_trace(long long *host, size_t bytes) {
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace), bytes) == hipSuccess ? 0 : 1;
}
#endif
