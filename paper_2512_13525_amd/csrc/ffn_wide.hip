// a5, bf16 path, slots with many requests: blocks of 128 request rows as tiled GEMMs.
//
// Janus Sec. 2.2: an expert's two GEMMs are memory-bound while few tokens visit it and turn
// compute-bound as the batch grows.  The streaming kernel (ffn_stream.hip) is built for the first
// regime: a slot with several blocks of rows streams its expert once per block.  In batches of
// thousands of tokens a slot that received more than 64 requests is therefore taken out of the
// streaming launch and handled here: its rows are cut into blocks of 128, and a workgroup computes 128 rows x 4 packed weight tiles
// (64 channels of SiLU(gate)*up in stage 1, 128 output channels in stage 2), so that the weights
// are fetched once per 128 rows and the token rows once per 4 tiles.
//
// Each of the 4 wavefronts owns one packed tile (two MFMA A fragments per K-step, read straight
// from global memory: the packed layout is the register image) and all 128 rows: 8 row tiles x 2
// accumulators.  Gate and up of a channel live in the same lane, so stage 1 needs no exchange
// between wavefronts.  The token rows (the B operand, shared by the 4 wavefronts) go through LDS:
// per K-tile of 64 columns the workgroup reads one 128-byte line of each row with whole-line
// loads (8 rows per instruction) into a double-buffered, XOR-swizzled 16 KiB tile, from which
// every wavefront reads the MFMA layout.  One barrier per K-tile; two K-tiles of both operands
// are in flight in registers (three workgroups fit a CU).
//
// A workgroup runs the whole K dimension of its tile, so these launches pay off only when a
// batch has enough wide blocks to fill the chip; the list header counts them and this kernel and
// the streaming kernel take the same decision from it (moe::ffn_gemm_on).
//
// Work comes from the same block list as the streaming launch (blocks of 64 rows): the entry
// whose first row is a multiple of 128 rows into a slot with more than 64 requests leads a wide
// block; every other entry leaves at once.  The two stages are two launches; the intermediate is
// row-major bf16 [request row][d_e] in the workspace.
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = moe::kWideWaves;
constexpr int kThreads = kWaves * MOE_WAVE;
constexpr int kLoadsB = 128 * 8 / kThreads;     // 16-byte pieces of the 128 x 128-byte token tile per thread
constexpr int kRows = 128;               // request rows of a wide block
constexpr int kRowTiles = kRows / 16;
constexpr int kRing = 2;                 // K-tiles of both operands in flight (register sets)
constexpr unsigned kPanelItems = 24;     // list entries (of 64 rows: 12 blocks of 128 rows) of a panel of workgroups
constexpr unsigned kPanelTiles = 8;      // workgroup tiles of a panel
constexpr unsigned kPanelSize = kPanelItems * kPanelTiles;

struct WideArgs {
    const char *B;                       // token operand: X (stage 1, rows through perm) or the intermediate (stage 2)
    const char *Wp;                      // packed weights: [C][ptiles][KS][2][64] fragments of 16 bytes
    const int32_t *blocks, *perm;
    const int *ctrl;                     // control region of the workspace (header word kCtrlWideMin)
    uint16_t *act;                       // stage-1 output [request row][out_stride]
    float *Yp;                           // stage-2 output [request row][out_stride]
    int ptiles, tiles, tiles_pad, KS;    // tiles = workgroup tiles of 4 packed tiles
    int tiles1, wide_min;                // workgroup tiles of stage 1 and the threshold of the on/off rule
    int k;
    uint32_t b_row_bytes;
    int out_stride;
};

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + __expf(-g)) * u; }

// One wide block.  UPPER: the block has more than 64 rows (all 8 row tiles are computed; otherwise
// only the lower 4), so the K loop has no data-dependent branch.
template <bool STAGE1, bool UPPER>
__device__ __forceinline__ void wide_block(const WideArgs &a, char (*lds)[kRows * 128], int tile, int slot, int row0, int m);

template <bool STAGE1>
__global__ __launch_bounds__(kThreads, kRing == 2 ? 3 : 2)
void ffn_wide_kernel(WideArgs a) {
    __shared__ __attribute__((aligned(16))) char lds[2][kRows * 128];
    // Workgroup ids go round-robin over the eight XCDs, each with an L2 of its own.  The (list entry, tile)
    // grid is cut into panels of kPanelItems entries x kPanelTiles tiles; a panel is a run of consecutive
    // workgroups of ONE XCD (about as many as the XCD holds at a time), so the tiles of a block share its
    // token rows and the sibling blocks of a slot share the expert's tiles in that L2 while they walk K
    // side by side.  Panels go to the XCDs in turn, the tile panels of the same entries first.
    const unsigned xcd = blockIdx.x & 7u, q = blockIdx.x >> 3;
    const unsigned panel = (q / kPanelSize) * 8u + xcd, r = q % kPanelSize;
    const unsigned tile_panels = static_cast<unsigned>(a.tiles + kPanelTiles - 1) / kPanelTiles;
    const int tile = static_cast<int>((panel % tile_panels) * kPanelTiles + r % kPanelTiles);
    const long long item_ll = static_cast<long long>(panel / tile_panels) * kPanelItems + r / kPanelTiles;
    if (tile >= a.tiles) return;
    const int4 *list = reinterpret_cast<const int4 *>(a.blocks);
    const int4 head = list[0];
    if (item_ll >= head.x) return;
    const int item = static_cast<int>(item_ll);
    const int wm_ws = a.ctrl[moe::kCtrlWideMin];                     // the workspace's threshold, 0 = default
    if (!moe::ffn_gemm_on(head, a.tiles1, wm_ws)) return;
    const int4 ent = list[1 + item];
    const int slot = ent.x, row0 = ent.y, hi = ent.z;
    const int lo = ent.w;                                            // first of the slot's rows
    // the leader of a wide block: more than 64 requests on the slot, first row a multiple of 128 into it
    if (hi - lo <= 64 || ((row0 - lo) & (kRows - 1)) != 0) return;
    const int m = hi - row0 < kRows ? hi - row0 : kRows;             // rows of this block
    if (m > 64) wide_block<STAGE1, true>(a, lds, tile, slot, row0, m);
    else wide_block<STAGE1, false>(a, lds, tile, slot, row0, m);
}

template <bool STAGE1, bool UPPER>
__device__ __forceinline__ void wide_block(const WideArgs &a, char (*lds)[kRows * 128], int tile, int slot, int row0, int m) {
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / MOE_WAVE), lane = tid % MOE_WAVE;
    int pt = tile * kWaves + wave;
    const bool pt_ok = pt < a.ptiles;
    pt = pt_ok ? pt : a.ptiles - 1;
    const char *w = a.Wp + (static_cast<size_t>(slot) * a.ptiles + pt) * a.KS * 2048 + lane * 16;

    // token rows this thread fetches: rows q*(kThreads/8) + tid/8, 16-byte chunk tid%8 of the line
    const char *bp[kLoadsB];
#pragma unroll
    for (int q = 0; q < kLoadsB; ++q) {
        int r = q * (kThreads / 8) + (tid >> 3);
        r = row0 + (r < m ? r : m - 1);
        const size_t src = STAGE1 ? static_cast<size_t>(a.perm[r] / a.k) : static_cast<size_t>(r);
        bp[q] = a.B + src * a.b_row_bytes + (tid & 7) * 16;
    }
    // LDS: row R at R*128, its 16-byte chunk c at ((c ^ ((R >> 1) & 7)) * 16): the 16 rows that one
    // fragment read touches then fall into 16 different bank groups (rows R and R+8 share R & 7)
    const uint32_t wr_lds = (tid >> 3) * 128 + (((tid & 7) ^ ((tid >> 4) & 7)) * 16);
    const uint32_t rd_row = (lane & 15) * 128, rd_sw = (lane >> 1) & 7, rd_g = lane >> 4;

    const int NT = (a.KS + 1) >> 1;                                  // K-tiles of two K-steps (the last may hold one); >= 1
    f32x4 acc[kRowTiles][2];
#pragma unroll
    for (int rt = 0; rt < kRowTiles; ++rt) { acc[rt][0] = f32x4{0.f, 0.f, 0.f, 0.f}; acc[rt][1] = acc[rt][0]; }
    // kRing K-tiles of both operands are in flight in a ring of register sets (K-tile i uses set
    // i % kRing and LDS buffer i % 2); loads past the last K-tile fetch the last one again, so the steady-state
    // loop has no branch around a load and the compiler counts outstanding loads exactly.
    bf16x8 breg[kRing][kLoadsB];
    bf16x8 areg[kRing][2][2];                                        // [set][K-step of the tile][fragment]
    const int last = NT - 1;

    // K-tile j: columns 64*j .. 64*j+63.  With an odd number of K-steps the last tile has only its
    // first half: its second K-step repeats the first (never multiplied) and chunks 4..7 of the
    // line, which lie past the row, repeat chunks 0..3.
#define MOE_WIDE_LOAD_A(set, j)                                                                  \
    do {                                                                                         \
        const int j_ = (j) < last ? (j) : last;                                                  \
        const int s0_ = 2 * j_, s1_ = 2 * j_ + 1 < a.KS ? 2 * j_ + 1 : 2 * j_;                   \
        areg[set][0][0] = *reinterpret_cast<const bf16x8 *>(w + static_cast<size_t>(s0_) * 2048);         \
        areg[set][0][1] = *reinterpret_cast<const bf16x8 *>(w + static_cast<size_t>(s0_) * 2048 + 1024);  \
        areg[set][1][0] = *reinterpret_cast<const bf16x8 *>(w + static_cast<size_t>(s1_) * 2048);         \
        areg[set][1][1] = *reinterpret_cast<const bf16x8 *>(w + static_cast<size_t>(s1_) * 2048 + 1024);  \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
#define MOE_WIDE_LOAD_B(set, j)                                                                  \
    do {                                                                                         \
        const int j_ = (j) < last ? (j) : last;                                                  \
        const size_t off_ = static_cast<size_t>(j_) * 128 - ((2 * j_ + 1 >= a.KS && (tid & 7) >= 4) ? 64 : 0); \
        _Pragma("unroll") for (int q = 0; q < kLoadsB; ++q)                                      \
            breg[set][q] = *reinterpret_cast<const bf16x8 *>(bp[q] + off_);                      \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
#define MOE_WIDE_STAGE(set)                                                                      \
    do {                                                                                         \
        _Pragma("unroll") for (int q = 0; q < kLoadsB; ++q)                                      \
            *reinterpret_cast<bf16x8 *>(lds[(set) & 1] + q * (kThreads * 16) + wr_lds) = breg[set][q];       \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
#define MOE_WIDE_MMA_HALF(set, ss, h)                                                            \
    do {                                                                                         \
        bf16x8 b_[4];                                                                            \
        _Pragma("unroll") for (int r4 = 0; r4 < 4; ++r4)                                         \
            b_[r4] = *reinterpret_cast<const bf16x8 *>(                                          \
                lds[(set) & 1] + ((h) * 4 + r4) * 2048 + rd_row + (((4 * (ss) + rd_g) ^ rd_sw) * 16)); \
        _Pragma("unroll") for (int r4 = 0; r4 < 4; ++r4) {                                       \
            acc[(h) * 4 + r4][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(areg[set][ss][0], b_[r4], acc[(h) * 4 + r4][0], 0, 0, 0); \
            acc[(h) * 4 + r4][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(areg[set][ss][1], b_[r4], acc[(h) * 4 + r4][1], 0, 0, 0); \
        }                                                                                        \
    } while (0)
    // rows past the block's last repeat that row (their results are not stored); the upper four row
    // tiles are skipped when the block has at most 64 rows
#define MOE_WIDE_MMA(set, full)                                                                  \
    do {                                                                                         \
        MOE_WIDE_MMA_HALF(set, 0, 0);                                                            \
        if constexpr (UPPER) MOE_WIDE_MMA_HALF(set, 0, 1);                                       \
        if (full) {                                                                              \
            MOE_WIDE_MMA_HALF(set, 1, 0);                                                        \
            if constexpr (UPPER) MOE_WIDE_MMA_HALF(set, 1, 1);                                   \
        }                                                                                        \
        asm volatile("" ::: "memory");                                                           \
    } while (0)
    // The LDS buffer written here was last read in the multiply of K-tile i-2, which every wavefront
    // finished before the barrier of K-tile i-1.  full: both K-steps of the tile exist (a literal, so
    // the multiply of a full tile is one straight run of LDS reads and MFMAs).
#define MOE_WIDE_STEP(set, i, full)                                                              \
    do {                                                                                         \
        MOE_WIDE_STAGE(set);                                                                     \
        MOE_WIDE_LOAD_B(set, (i) + kRing);                                                       \
        __syncthreads();                                                                         \
        MOE_WIDE_MMA(set, full);                                                                 \
        MOE_WIDE_LOAD_A(set, (i) + kRing);                                                       \
    } while (0)

    const int n_full = a.KS >> 1;                                    // K-tiles with both K-steps
    int i = 0;
    if constexpr (kRing == 4) {
        MOE_WIDE_LOAD_A(0, 0); MOE_WIDE_LOAD_B(0, 0);
        MOE_WIDE_LOAD_A(1, 1); MOE_WIDE_LOAD_B(1, 1);
        MOE_WIDE_LOAD_A(2, 2); MOE_WIDE_LOAD_B(2, 2);
        MOE_WIDE_LOAD_A(3, 3); MOE_WIDE_LOAD_B(3, 3);
        for (; i + 4 <= n_full; i += 4) {
            MOE_WIDE_STEP(0, i, true);
            MOE_WIDE_STEP(1, i + 1, true);
            MOE_WIDE_STEP(2, i + 2, true);
            MOE_WIDE_STEP(3, i + 3, true);
        }
        const int rem = n_full - i;                                  // 0 .. 3 full K-tiles left
        if (rem > 0) MOE_WIDE_STEP(0, i, true);
        if (rem > 1) MOE_WIDE_STEP(1, i + 1, true);
        if (rem > 2) MOE_WIDE_STEP(2, i + 2, true);
        if (a.KS & 1) {                                              // the half tile of an odd number of K-steps
            switch (rem) {
                case 0: MOE_WIDE_STEP(0, n_full, false); break;
                case 1: MOE_WIDE_STEP(1, n_full, false); break;
                case 2: MOE_WIDE_STEP(2, n_full, false); break;
                default: MOE_WIDE_STEP(3, n_full, false); break;
            }
        }
    } else {
        static_assert(kRing == 2 || kRing == 4, "the K loop is written out for rings of 2 and 4");
        MOE_WIDE_LOAD_A(0, 0); MOE_WIDE_LOAD_B(0, 0);
        MOE_WIDE_LOAD_A(1, 1); MOE_WIDE_LOAD_B(1, 1);
        for (; i + 2 <= n_full; i += 2) {
            MOE_WIDE_STEP(0, i, true);
            MOE_WIDE_STEP(1, i + 1, true);
        }
        const int rem = n_full - i;                                  // 0 .. 1
        if (rem > 0) MOE_WIDE_STEP(0, i, true);
        if (a.KS & 1) {
            if (rem == 0) MOE_WIDE_STEP(0, n_full, false);
            else MOE_WIDE_STEP(1, n_full, false);
        }
    }
#undef MOE_WIDE_LOAD_A
#undef MOE_WIDE_LOAD_B
#undef MOE_WIDE_STAGE
#undef MOE_WIDE_MMA
#undef MOE_WIDE_MMA_HALF
#undef MOE_WIDE_STEP

    if (!pt_ok) return;
    // lane l holds, per row tile, 4 consecutive channels (l/16)*4.. of row (l%16) of the tile
#pragma unroll
    for (int rt = 0; rt < kRowTiles; ++rt) {
        const int r = rt * 16 + (lane & 15);
        if (r >= m) continue;
        const size_t row = static_cast<size_t>(row0 + r);
        if (STAGE1) {
            const f32x4 g = acc[rt][0], u = acc[rt][1];
            const uint64_t o = static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(g[0], u[0]))) |
                               static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(g[1], u[1]))) << 16 |
                               static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(g[2], u[2]))) << 32 |
                               static_cast<uint64_t>(moe::f32_to_bf16(silu_mul(g[3], u[3]))) << 48;
            *reinterpret_cast<uint64_t *>(a.act + row * a.out_stride + pt * 16 + (lane >> 4) * 4) = o;
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h)
                *reinterpret_cast<f32x4 *>(a.Yp + row * a.out_stride + pt * 32 + h * 16 + (lane >> 4) * 4) = acc[rt][h];
        }
    }
}

// Workgroups of a launch over `items` list entries and `tiles` workgroup tiles: whole panels, eight at a time.
long long wide_grid(long long items, int tiles) {
    const long long panels = ((items + kPanelItems - 1) / kPanelItems) * ((tiles + kPanelTiles - 1) / kPanelTiles);
    return (panels + 7) / 8 * 8 * kPanelSize;
}

}  // namespace

namespace moe {

// Both stages for every wide block of the list (two launches sized for the largest possible number
// of blocks; workgroups that find no wide block leave after three scalar loads).
int launch_ffn_wide(const void *X, const void *W13p, const void *W2p, int T, int k, int C, int d_h, int d_e,
                    const int32_t *blocks, const int32_t *perm, const int *ctrl, uint16_t *act_rows,
                    float *Yp, hipStream_t st) {
    const long long items = ffn_max_blocks(T, k, C);
    WideArgs a;
    a.blocks = blocks; a.perm = perm; a.ctrl = ctrl; a.act = act_rows; a.Yp = Yp; a.k = k;
    // stage 1
    a.B = static_cast<const char *>(X); a.Wp = static_cast<const char *>(W13p);
    a.ptiles = d_e / 16; a.KS = d_h / 32; a.b_row_bytes = static_cast<uint32_t>(d_h) * 2; a.out_stride = d_e;
    a.tiles = (a.ptiles + kWaves - 1) / kWaves; a.tiles_pad = (a.tiles + 7) / 8 * 8; a.tiles1 = a.tiles; a.wide_min = 0;
    long long grid = wide_grid(items, a.tiles);
    if (grid > 0x7fffffffLL) return MOE_ESHAPE;
    hipLaunchKernelGGL(ffn_wide_kernel<true>, dim3(static_cast<unsigned>(grid)), dim3(kThreads), 0, st, a);
    // stage 2
    a.B = reinterpret_cast<const char *>(act_rows); a.Wp = static_cast<const char *>(W2p);
    a.ptiles = d_h / 32; a.KS = d_e / 32; a.b_row_bytes = static_cast<uint32_t>(d_e) * 2; a.out_stride = d_h;
    a.tiles = (a.ptiles + kWaves - 1) / kWaves; a.tiles_pad = (a.tiles + 7) / 8 * 8;
    grid = wide_grid(items, a.tiles);
    if (grid > 0x7fffffffLL) return MOE_ESHAPE;
    hipLaunchKernelGGL(ffn_wide_kernel<false>, dim3(static_cast<unsigned>(grid)), dim3(kThreads), 0, st, a);
    return MOE_OK;
}

}  // namespace moe
