// a0-a4 in ONE launch: gating selection for all tokens, then Alg. 1 and this instance's
// dispatch (Janus Sec. 3.4, workflow Steps 0-4).  At decode sizes each of these steps is a few
// microseconds of work behind a launch of about the same cost, so three launches become one.
//
// Every workgroup routes 4, 8 or 16 tokens (one per wavefront; the fewer, the smaller the batch:
// launch_front) and publishes their expert ids with agent-scope stores; the workgroup that finishes last (an atomic ticket, nobody waits) then
// runs Alg. 1 and the counting sort on its own, reading the ids with agent-scope loads because
// they were written on other XCDs.
//
// The gated variants start one step earlier (Sec. 3.3: gating runs on the MoE side, from the
// complete activations): the logits are the router's linear layer X * W_r^T (+ bias), computed
// in the same launch.  A workgroup owns (16 tokens) x (16 experts) of the logits: its 16
// wavefronts split the hidden dimension, each accumulates one 16x16 MFMA tile over its share,
// and the partial tiles are summed in LDS in wavefront order.  The workgroup that completes a
// token group (a ticket per group) routes its 16 tokens from the logits the others published.
#include "dispatch_dev.h"

namespace {

struct FrontArgs {
    const float *logits;
    int T, E, k;
    moe_route_cfg cfg;
    int32_t *ids;
    float *w;
    moe::SchedTables tb;
    int n_inst, C, n_words, g_self;
    int32_t *rid, *act_rep, *load, *slot_count, *slot_off, *perm, *pos, *blocks;
    int32_t *ticket;
    int block_rows;
    // gated variants: logits = X * Wr^T (+ bias) are computed here and written to `logits_out`
    const uint16_t *X, *Wr;              // bf16 [T,d_h], [E,d_h]
    const float *bias;                   // [E] or null
    float *logits_out;                   // [T,E]
    int d_h, n_tiles;                    // n_tiles = ceil(E/16) expert tiles
    int tail;                            // 0: stop after the gating selection
    // batches too large for the one-workgroup tail (launch from logits only): the routing workgroups
    // raise the activated experts in act_bits, the last one runs Step 2 of Alg. 1 from them, and two
    // further launches (front_count_kernel, front_scatter_kernel) rewrite and sort the requests in chunks
    uint32_t *act_bits;                  // [kBitWords], zero between calls; null = one-workgroup tail
    int32_t *hist;                       // [n_chunks][C]
    int chunk_pairs, n_chunks;
    int tok_per_wg;                      // launch from logits: wavefronts of a workgroup that route a token (4, 8 or 16)
};
constexpr int kBitWords = MOE_MAX_EXPERTS / 32;
constexpr int kChunkPairs = 2048;

constexpr int kGateUnroll = 4;
constexpr int kGateDepth = 4;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Logits of token group tg (16 tokens) against expert tile j (16 experts).  MFMA 16x16x32: the
// router rows are the A operand (lane l: expert l%16, 8 columns at (l/16)*8 of the K-step), the
// token rows the B operand (same shape), and the D tile leaves lane l with experts (l/16)*4..+3
// of token l%16.  Rows past T or E repeat the last valid row and are not stored.
//
// This wavefront's share of the sum, operands read straight into the MFMA layout: every lane
// requests its own 16 bytes of its own row, four requests per 64 bytes.  Used when the hidden
// size is not a multiple of 64.
__device__ __forceinline__ f32x4 gate_acc_steps(const FrontArgs &a, int tg, int j, int wave, int lane) {
    const int KS = a.d_h / 32;
    const int per = (KS + moe::kFrontWaves - 1) / moe::kFrontWaves;
    const int k0 = wave * per;
    const int k1 = k0 + per < KS ? k0 + per : KS;
    int tok = tg * 16 + (lane & 15);
    tok = tok < a.T ? tok : a.T - 1;
    int e = j * 16 + (lane & 15);
    e = e < a.E ? e : a.E - 1;
    const char *xb = reinterpret_cast<const char *>(a.X) + (static_cast<size_t>(tok) * a.d_h + (lane >> 4) * 8) * 2;
    const char *wb = reinterpret_cast<const char *>(a.Wr) + (static_cast<size_t>(e) * a.d_h + (lane >> 4) * 8) * 2;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    // kGateUnroll K-steps of both operands in flight; steps past the share load the last valid step
    // again and multiply by zero, so the loop has no tail
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int kk = k0; kk < k1; kk += kGateUnroll) {
        bf16x8 av[kGateUnroll], bv[kGateUnroll];
#pragma unroll
        for (int u = 0; u < kGateUnroll; ++u) {
            const int q = kk + u < k1 ? kk + u : k1 - 1;
            av[u] = *reinterpret_cast<const bf16x8 *>(wb + q * 64);
            bv[u] = *reinterpret_cast<const bf16x8 *>(xb + q * 64);
        }
#pragma unroll
        for (int u = 0; u < kGateUnroll; ++u)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[u], kk + u < k1 ? bv[u] : zero, acc, 0, 0, 0);
    }
    return acc;
}

// The same share with whole-line reads (hidden size a multiple of 64): a super-step is 64 columns =
// one 128-byte line of each of the 16 + 16 rows; a load instruction fetches 8 whole lines (lane l:
// row l/8, 16-byte chunk l%8), a quarter of the requests of the direct form, and the MFMA layout
// comes from a round trip through a wave-private 4 KiB LDS tile (chunks XOR-swizzled by row so
// that the row-major writes and the column-wise reads both spread over the banks).  Wavefront w
// takes super-steps w, w+16, ...; kGateDepth of them are in flight.
__device__ __forceinline__ f32x4 gate_acc_lines(const FrontArgs &a, int tg, int j, char *stage, int wave, int lane) {
    const int SS = a.d_h / 64;
    const int n = (SS - wave + moe::kFrontWaves - 1) / moe::kFrontWaves;
    char *st = stage + wave * 4096;                                  // [router rows | token rows][16 rows][128 bytes]
    const char *wp[2], *xp[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        int e = j * 16 + h * 8 + (lane >> 3);
        e = e < a.E ? e : a.E - 1;
        int t = tg * 16 + h * 8 + (lane >> 3);
        t = t < a.T ? t : a.T - 1;
        wp[h] = reinterpret_cast<const char *>(a.Wr) + static_cast<size_t>(e) * a.d_h * 2 + (lane & 7) * 16;
        xp[h] = reinterpret_cast<const char *>(a.X) + static_cast<size_t>(t) * a.d_h * 2 + (lane & 7) * 16;
    }
    // LDS: row R of an operand at R*128, its 16-byte chunk c at ((c ^ (R & 7)) * 16)
    const uint32_t wr_lds = ((lane >> 3) * 128) + (((lane & 7) ^ (lane >> 3)) * 16);
    const uint32_t rd_row = (lane & 15) * 128, rd_sw = lane & 7, rd_g = lane >> 4;
    bf16x8 ld[kGateDepth][4];
#define MOE_GATE_LOAD(d, i)                                                                      \
    do {                                                                                         \
        const size_t off_ = static_cast<size_t>(wave + moe::kFrontWaves * (i)) * 128;            \
        ld[d][0] = *reinterpret_cast<const bf16x8 *>(wp[0] + off_);                              \
        ld[d][1] = *reinterpret_cast<const bf16x8 *>(wp[1] + off_);                              \
        ld[d][2] = *reinterpret_cast<const bf16x8 *>(xp[0] + off_);                              \
        ld[d][3] = *reinterpret_cast<const bf16x8 *>(xp[1] + off_);                              \
    } while (0)
#pragma unroll
    for (int d = 0; d < kGateDepth; ++d)
        if (d < n) MOE_GATE_LOAD(d, d);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < n; i += kGateDepth) {
#pragma unroll
        for (int d = 0; d < kGateDepth; ++d) {
            if (i + d < n) {                                         // wave-uniform
#pragma unroll
                for (int q = 0; q < 4; ++q) *reinterpret_cast<bf16x8 *>(st + q * 1024 + wr_lds) = ld[d][q];
                asm volatile("" ::: "memory");
                if (i + d + kGateDepth < n) MOE_GATE_LOAD(d, i + d + kGateDepth);
#pragma unroll
                for (int ss = 0; ss < 2; ++ss) {
                    const uint32_t o = rd_row + (((4 * ss + rd_g) ^ rd_sw) * 16);
                    const bf16x8 av = *reinterpret_cast<const bf16x8 *>(st + o);
                    const bf16x8 bv = *reinterpret_cast<const bf16x8 *>(st + 2048 + o);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, acc, 0, 0, 0);
                }
                asm volatile("" ::: "memory");
            }
        }
    }
#undef MOE_GATE_LOAD
    return acc;
}

// lds: 64 KiB.  The partial tiles of the 16 wavefronts are summed in wavefront order.
__device__ __forceinline__ void gate_tile(const FrontArgs &a, int tg, int j, char *lds, int wave, int lane) {
    // the bias of this lane's four experts, fetched up front so that the stores at the end follow
    // one another without a load (and its wait for the previous store) in between
    float bias[4] = {0.f, 0.f, 0.f, 0.f};
    if (a.bias && threadIdx.x < MOE_WAVE) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ee = j * 16 + (lane >> 4) * 4 + i;
            bias[i] = a.bias[ee < a.E ? ee : a.E - 1];
        }
    }
    f32x4 acc;
    if (a.d_h % 64 == 0) {
        acc = gate_acc_lines(a, tg, j, lds, wave, lane);
        __syncthreads();                                             // the staging tiles give way to the partial tiles
    } else {
        acc = gate_acc_steps(a, tg, j, wave, lane);
    }
    f32x4 *part = reinterpret_cast<f32x4 *>(lds);
    part[wave * MOE_WAVE + lane] = acc;
    __syncthreads();
    if (threadIdx.x < MOE_WAVE) {
        f32x4 s = part[lane];
#pragma unroll
        for (int w = 1; w < moe::kFrontWaves; ++w) s += part[w * MOE_WAVE + lane];
        const int t = tg * 16 + (lane & 15);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ee = j * 16 + (lane >> 4) * 4 + i;
            if (t < a.T && ee < a.E)
                __hip_atomic_store(a.logits_out + static_cast<size_t>(t) * a.E + ee, s[i] + bias[i],
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Decode-size tail (up to kRegPairs requests): Alg. 1 and the counting sort with every request id
// held in registers.  Wavefront w owns requests [w*gpw*64, (w+1)*gpw*64), the mapping the sort needs,
// so the ids are read from memory exactly once (one round trip together with the layout tables)
// and everything after that runs out of LDS and registers.
constexpr int kGpwMax = 8;                                            // 64-request groups per wavefront
constexpr int kRegPairs = moe::kFrontWaves * kGpwMax * MOE_WAVE;      // 8192
constexpr int kSlotOfLds = 8192;                                      // E*n_inst entries of slot_of kept in LDS

// Layout tables one thread fetches at kernel entry (every workgroup does, only the last one uses
// them): their latency hides behind the routing instead of following the ticket.
struct TablePrefetch {
    uint64_t host_mask, multi_mask, single_mask;
    int32_t single_rid;
    uint4 slot_of;                                                    // 8 int16 entries
};

__device__ __forceinline__ TablePrefetch prefetch_tables(const FrontArgs &a) {
    TablePrefetch t{};
    const int tid = threadIdx.x;
    if (tid < a.E) { t.host_mask = a.tb.host_mask[tid]; t.single_rid = a.tb.single_rid[tid]; }
    if (tid < a.n_words) t.multi_mask = a.tb.multi_mask[tid];
    if (tid < a.n_inst * a.n_words) t.single_mask = a.tb.single_mask[tid];
    // the table is padded to a multiple of 256 bytes, so the last 16-byte read stays inside it
    if (tid * 8 < a.E * a.n_inst) t.slot_of = reinterpret_cast<const uint4 *>(a.tb.slot_of)[tid];
    return t;
}

struct SmallShared {
    moe::SchedShared sched;
    moe::PermShared perm;
    alignas(16) int16_t slot_of[kSlotOfLds];
};

__device__ __forceinline__ void front_tail_small(const FrontArgs &a, SmallShared &sh, int n_pairs,
                                                 const TablePrefetch &tp) {
    const int tid = threadIdx.x;
    const int wave = tid / MOE_WAVE, lane = tid % MOE_WAVE;
    const int E = a.E, n_inst = a.n_inst, C = a.C, n_words = a.n_words;
    const int n_groups = (n_pairs + MOE_WAVE - 1) / MOE_WAVE;
    const int gpw = (n_groups + moe::kFrontWaves - 1) / moe::kFrontWaves;   // <= kGpwMax

    // ---- one round trip: request ids (written by other workgroups: agent-scope loads) and tables
    int id[kGpwMax];
#pragma unroll
    for (int g = 0; g < kGpwMax; ++g) {
        const int p = (wave * gpw + g) * MOE_WAVE + lane;
        id[g] = (g < gpw && p < n_pairs) ? __hip_atomic_load(a.ids + p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : -1;
    }
    // E, n_words, n_inst*n_words <= 1024 threads and E*n_inst <= 8*1024: one element each
    if (tid < E) {
        sh.sched.flag[tid] = 0u;
        sh.sched.host_mask[tid] = tp.host_mask;
        sh.sched.single_rid[tid] = tp.single_rid;
    }
    if (tid < n_words) sh.sched.multi_mask[tid] = tp.multi_mask;
    if (tid < n_inst * n_words) sh.sched.single_mask[tid] = tp.single_mask;
    if (tid * 8 < E * n_inst) reinterpret_cast<uint4 *>(sh.slot_of)[tid] = tp.slot_of;
    for (int i = tid; i < moe::kFrontWaves * MOE_MAX_SLOTS; i += moe::kFrontThreads) (&sh.perm.cnt[0][0])[i] = 0;
    __syncthreads();

    // ---- Step 1
#pragma unroll
    for (int g = 0; g < kGpwMax; ++g)
        if (id[g] >= 0) sh.sched.flag[id[g]] = 1u;
    __syncthreads();

    // ---- Step 2 (first wavefront), as in aebs_block but with slot_of in LDS
    if (tid < MOE_WAVE) {
        int load = 0;
        for (int w = 0; w < n_words; ++w) {
            const int e = w * 64 + lane;
            const uint64_t act = __ballot(e < E && sh.sched.flag[e] != 0u);
            if (lane < n_inst) load += __popcll(act & sh.sched.single_mask[lane * n_words + w]);
        }
        for (int w = 0; w < n_words; ++w) {
            const int e = w * 64 + lane;
            const uint64_t act = __ballot(e < E && sh.sched.flag[e] != 0u);
            const uint64_t hm = e < E ? sh.sched.host_mask[e] : 0ull;
            uint64_t todo = act & moe::readfirstlane_u64(sh.sched.multi_mask[w]);
            int chosen = -1;
            while (todo) {
                const int b = __builtin_ctzll(todo);
                todo &= todo - 1;
                uint64_t hosts = moe::readlane_u64(hm, b);
                int best_g = __builtin_ctzll(hosts);
                int best_load = __builtin_amdgcn_readlane(load, best_g);
                hosts &= hosts - 1;
                while (hosts) {                         // ascending instance id: strict '<' keeps the lowest on ties
                    const int h = __builtin_ctzll(hosts);
                    hosts &= hosts - 1;
                    const int l = __builtin_amdgcn_readlane(load, h);
                    if (l < best_load) { best_load = l; best_g = h; }
                }
                if (lane == best_g) load += 1;
                if (lane == b) chosen = best_g;
            }
            if (e < E) {
                int rep = -1;
                if ((act >> lane) & 1ull) {
                    if (chosen >= 0) rep = chosen * C + sh.slot_of[e * n_inst + chosen];
                    else rep = sh.sched.single_rid[e];
                }
                sh.sched.rep[e] = rep;
                a.act_rep[e] = rep;
            }
        }
        if (lane < n_inst) a.load[lane] = load;
    }
    __syncthreads();

    // ---- Step 3 and pass A of the sort
    const int rid_lo = a.g_self * C;
    int sl[kGpwMax];                                                  // local slot, or -1
#pragma unroll
    for (int g = 0; g < kGpwMax; ++g) {
        sl[g] = -1;
        if (id[g] >= 0) {
            const int r = sh.sched.rep[id[g]];
            a.rid[(wave * gpw + g) * MOE_WAVE + lane] = r;
            const int s = r - rid_lo;
            if (s >= 0 && s < C) { sl[g] = s; atomicAdd(&sh.perm.cnt[wave][s], 1); }
        }
    }
    __syncthreads();
    for (int s = tid; s < C; s += moe::kFrontThreads) {
        int run = 0;
#pragma unroll
        for (int w = 0; w < moe::kFrontWaves; ++w) {
            const int c = sh.perm.cnt[w][s];
            sh.perm.cnt[w][s] = run;
            run += c;
        }
        sh.perm.total[s] = run;
        a.slot_count[s] = run;
    }
    __syncthreads();
    if (wave == 0) moe::scan_slots(sh.perm, C, a.block_rows, a.slot_off, lane);
    __syncthreads();
    moe::list_blocks(sh.perm, C, a.block_rows, a.blocks);

    // ---- pass B
    if (C <= MOE_WAVE) {
        // the wavefront's running base of slot s lives in lane s: the loop over a group's slots reads
        // and bumps it with scalar-indexed lane accesses, no LDS round trip per slot
        int base_reg = lane < C ? sh.perm.cnt[wave][lane] + sh.perm.off[lane] : 0;
#pragma unroll
        for (int g = 0; g < kGpwMax; ++g) {
            if (g < gpw) {                                            // wave-uniform
                const int p = (wave * gpw + g) * MOE_WAVE + lane;
                const int s = sl[g];
                const bool local = s >= 0;
                int row = -1;
                uint64_t todo = __ballot(local);
                while (todo) {
                    const int lead = __builtin_ctzll(todo);
                    const int s0 = __builtin_amdgcn_readlane(s, lead);
                    const uint64_t same = __ballot(local && s == s0);
                    const int b = __builtin_amdgcn_readlane(base_reg, s0);
                    if (local && s == s0) row = b + __popcll(same & moe::lanemask_lt());
                    if (lane == s0) base_reg += __popcll(same);
                    todo &= ~same;
                }
                if (p < n_pairs) {
                    a.pos[p] = row;
                    if (local) a.perm[row] = p;
                }
            }
        }
        return;
    }
    volatile int *base = &sh.perm.cnt[wave][0];
#pragma unroll
    for (int g = 0; g < kGpwMax; ++g) {
        if (g < gpw) {                                                // wave-uniform
            const int p = (wave * gpw + g) * MOE_WAVE + lane;
            const int s = sl[g];
            const bool local = s >= 0;
            int row = -1;
            uint64_t todo = __ballot(local);
            while (todo) {
                const int lead = __builtin_ctzll(todo);
                const int s0 = __builtin_amdgcn_readlane(s, lead);
                const uint64_t same = __ballot(local && s == s0);
                const int b = base[s0] + sh.perm.off[s0];
                if (local && s == s0) row = b + __popcll(same & moe::lanemask_lt());
                __builtin_amdgcn_wave_barrier();
                if (lane == lead) base[s0] += __popcll(same);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                todo &= ~same;
            }
            if (p < n_pairs) {
                a.pos[p] = row;
                if (local) a.perm[row] = p;
            }
        }
    }
}

template <int VPL, bool GATE>
__global__ __launch_bounds__(moe::kFrontThreads)
void front_kernel(FrontArgs a) {
    // the phases run one after another, so their LDS overlays
    union Shared {
        float row[moe::kFrontWaves][VPL * MOE_WAVE];
        moe::SchedShared sched;
        moe::PermShared perm;
        SmallShared small;
        char gate[moe::kFrontWaves * 4096];                           // gated variants: staging tiles, then partial tiles
    };
    __shared__ Shared sh;
    __shared__ int s_last;
    __shared__ uint32_t s_bits[kBitWords];                            // experts this workgroup's tokens selected

    const int wave = threadIdx.x / MOE_WAVE;
    const int lane = moe::lane_id();
    const int n_pairs = a.T * a.k;
    const bool small = n_pairs <= kRegPairs && a.E * a.n_inst <= kSlotOfLds;
    TablePrefetch tp{};
    int expected = static_cast<int>(gridDim.x);                       // arrivals that complete the selection
    if constexpr (GATE) {
        if (a.tail && small) tp = prefetch_tables(a);
        expected = a.T > 0 ? (a.T + 15) / 16 : 1;
        if (a.T > 0) {
            // workgroups go to the 8 XCDs round-robin: all expert tiles of a token group run on one XCD,
            // so each L2 reads an eighth of the activations (and the whole router matrix)
            const int r = blockIdx.x / 8;
            const int tg = blockIdx.x % 8 + 8 * (r / a.n_tiles), j = r % a.n_tiles;
            if (tg * 16 >= a.T) return;
            gate_tile(a, tg, j, sh.gate, wave, lane);
            __syncthreads();                                          // the partial tiles give way to the logits rows
            // the group's ticket must not overtake the logits
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (threadIdx.x == 0) {
                int32_t *grp = a.ticket + 1 + tg;
                const int old = __hip_atomic_fetch_add(grp, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_last = old == a.n_tiles - 1;
                if (s_last) __hip_atomic_store(grp, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __syncthreads();
            if (!s_last) return;
            const int t = tg * 16 + wave;
            if (t < a.T) {
                float *row = sh.row[wave];
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    const int e = lane + i * MOE_WAVE;
                    row[e] = e < a.E ? __hip_atomic_load(a.logits_out + static_cast<size_t>(t) * a.E + e, __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT)
                                     : 0.0f;
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                moe::route_token<VPL, true, true>(row, a.E, a.k, a.cfg, row, lane,
                                                  a.ids + static_cast<size_t>(t) * a.k, a.w + static_cast<size_t>(t) * a.k);
            }
        }
        if (!a.tail) return;
    } else {
        if (small) tp = prefetch_tables(a);
        if (a.act_bits) {
            if (threadIdx.x < kBitWords) s_bits[threadIdx.x] = 0u;
            __syncthreads();
        }
        // small batches route on a few wavefronts per workgroup (one or two per SIMD instead of four),
        // spread over more CUs: the selection is a long chain of cross-lane steps that four wavefronts
        // of one SIMD would take turns at
        const int t = blockIdx.x * a.tok_per_wg + wave;
        if (wave < a.tok_per_wg && t < a.T) {
            moe::route_token<VPL, true>(a.logits + static_cast<size_t>(t) * a.E, a.E, a.k, a.cfg, sh.row[wave], lane,
                                        a.ids + static_cast<size_t>(t) * a.k, a.w + static_cast<size_t>(t) * a.k,
                                        a.act_bits ? s_bits : nullptr);
        }
        if (a.act_bits) {
            // Step 1 of Alg. 1, spread over the routing workgroups: one atomic per non-empty word
            __syncthreads();
            if (threadIdx.x < kBitWords && s_bits[threadIdx.x])
                __hip_atomic_fetch_or(a.act_bits + threadIdx.x, s_bits[threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // a workgroup barrier does not wait for global stores: the ticket must not overtake the ids
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const int old = __hip_atomic_fetch_add(a.ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = old == expected - 1;
        if (s_last) __hip_atomic_store(a.ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
    }
    __syncthreads();
    if (!s_last) return;

    if (small) {
        front_tail_small(a, sh.small, n_pairs, tp);
        return;
    }
    if (a.act_bits) {
        // Step 2 from the bitset the routing workgroups left; Step 3 and the sort follow in two launches
        moe::aebs_stage_tables(a.tb, sh.sched, a.E, a.n_inst, a.n_words);
        for (int e = threadIdx.x; e < a.E; e += moe::kFrontThreads) {
            const uint32_t word = __hip_atomic_load(a.act_bits + (e >> 5), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sh.sched.flag[e] = (word >> (e & 31)) & 1u;
        }
        __syncthreads();
        if (threadIdx.x < kBitWords)                                  // ready for the next call
            __hip_atomic_store(a.act_bits + threadIdx.x, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        moe::aebs_select(a.tb, sh.sched, a.E, a.n_inst, a.C, a.n_words, a.act_rep, a.load);
        return;
    }
    const int vec_ok = ((reinterpret_cast<uintptr_t>(a.ids) | reinterpret_cast<uintptr_t>(a.rid)) & 15) == 0;
    moe::aebs_block(a.tb, sh.sched, a.E, a.n_inst, a.C, a.n_words, a.ids, n_pairs, vec_ok, true,
                    a.rid, a.act_rep, a.load);
    // rid is re-read below by other wavefronts of this workgroup
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    moe::permute_block(sh.perm, a.rid, n_pairs, a.g_self, a.C, a.slot_count, a.slot_off, a.perm, a.pos, a.blocks, a.block_rows);
}

// Step 3 of Alg. 1 for one chunk of requests and the chunk's per-slot counts.
__global__ __launch_bounds__(moe::kFrontThreads)
void front_count_kernel(FrontArgs a) {
    __shared__ moe::PermShared sh;
    __shared__ int32_t rep[MOE_MAX_EXPERTS];
    for (int e = threadIdx.x; e < a.E; e += moe::kFrontThreads) rep[e] = a.act_rep[e];
    __syncthreads();
    const int n_pairs = a.T * a.k;
    const int p0 = blockIdx.x * a.chunk_pairs, p1 = min(n_pairs, p0 + a.chunk_pairs);
    moe::count_chunk(sh, rep, a.ids, a.rid, p0, p1, a.g_self, a.C, a.hist + blockIdx.x * a.C);
}

// The stable sort of one chunk into its places, from the counts of all chunks.
__global__ __launch_bounds__(moe::kFrontThreads)
void front_scatter_kernel(FrontArgs a) {
    __shared__ moe::PermShared sh;
    __shared__ int lower[MOE_MAX_SLOTS];
    const int n_pairs = a.T * a.k;
    const int p0 = blockIdx.x * a.chunk_pairs, p1 = min(n_pairs, p0 + a.chunk_pairs);
    moe::scatter_chunk(sh, lower, a.rid, p0, p1, blockIdx.x, a.n_chunks, a.hist, a.g_self, a.C, a.slot_count, a.slot_off,
                       a.perm, a.pos, a.blocks, a.block_rows);
}

#ifndef MOE_TPW
#define MOE_TPW 0
#endif
template <int VPL, bool GATE>
int launch_front(const FrontArgs &a_in, const char *what, hipStream_t st) {
    FrontArgs a = a_in;
    // every routing workgroup takes a ticket from one counter: keep them to about a hundred
    a.tok_per_wg = MOE_TPW ? MOE_TPW : a.T <= 512 ? 4 : a.T <= 1024 ? 8 : moe::kFrontWaves;
    int blocks = 1;
    if (a.T > 0) blocks = GATE ? (a.T + 127) / 128 * 8 * a.n_tiles : (a.T + a.tok_per_wg - 1) / a.tok_per_wg;
    hipLaunchKernelGGL((front_kernel<VPL, GATE>), dim3(blocks), dim3(moe::kFrontThreads), 0, st, a);
    if (!GATE && a.act_bits) {
        hipLaunchKernelGGL(front_count_kernel, dim3(a.n_chunks), dim3(moe::kFrontThreads), 0, st, a);
        hipLaunchKernelGGL(front_scatter_kernel, dim3(a.n_chunks), dim3(moe::kFrontThreads), 0, st, a);
    }
    return moe::check_launch(what);
}

// Batches whose requests do not fit the registers of one workgroup (or whose layout table does not
// fit its LDS) take the chunked tail.
bool front_is_large(const moe_placement_t *pl, int T, int k) {
    return static_cast<long long>(T) * k > kRegPairs || pl->E * pl->n_inst > kSlotOfLds;
}

template <bool GATE>
int launch_front_for(const FrontArgs &a, const char *what, hipStream_t st) {
    const int vpl = (a.E + MOE_WAVE - 1) / MOE_WAVE;
    if (vpl <= 1) return launch_front<1, GATE>(a, what, st);
    if (vpl <= 2) return launch_front<2, GATE>(a, what, st);
    if (vpl <= 4) return launch_front<4, GATE>(a, what, st);
    if (vpl <= 8) return launch_front<8, GATE>(a, what, st);
    return launch_front<16, GATE>(a, what, st);
}

int check_selection(int T, int E, int k, const moe_route_cfg *cfg) {
    if (!cfg || T < 0 || E < 1 || k < 1 || k > E) return MOE_EINVAL;
    if (E > MOE_MAX_EXPERTS || k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (static_cast<long long>(T) * k > 0x7fffffffLL) return MOE_ESHAPE;
    if (cfg->mode != MOE_ROUTE_SOFTMAX && cfg->mode != MOE_ROUTE_SIGMOID_GROUP) return MOE_EINVAL;
    if (cfg->mode == MOE_ROUTE_SIGMOID_GROUP) {
        if (cfg->n_group < 1 || cfg->topk_group < 1 || cfg->topk_group > cfg->n_group) return MOE_EINVAL;
        if (cfg->n_group > 64 || E % cfg->n_group != 0 || E / cfg->n_group < 2) return MOE_ESHAPE;
        if (k > cfg->topk_group * (E / cfg->n_group)) return MOE_EINVAL;
    }
    return MOE_OK;
}

// the gate's operands: bf16 rows of d_h elements read 16 bytes at a time
int check_gate(const void *X, const void *Wr, const float *bias, const float *logits, int T, int E, int d_h) {
    if (d_h < 32 || d_h % 32 != 0) return MOE_ESHAPE;
    if (static_cast<long long>(T) * E > 0x7fffffffLL) return MOE_ESHAPE;
    if (!Wr || !moe::aligned(Wr, 16) || !moe::aligned(bias, 4)) return MOE_EINVAL;
    if (T > 0 && (!X || !logits || !moe::aligned(X, 16) || !moe::aligned(logits, 4))) return MOE_EINVAL;
    return MOE_OK;
}

int fill_tail(FrontArgs &a, const moe_placement_t *pl, int g_self, int T, int32_t *rid_dev, int32_t *act_rep_dev,
              int32_t *load_dev, int32_t *slot_count_dev, int32_t *slot_off_dev, int32_t *perm_dev, int32_t *pos_dev,
              int32_t *blocks_dev) {
    if (g_self < 0 || g_self >= pl->n_inst) return MOE_EINVAL;
    if (!act_rep_dev || !load_dev || !slot_count_dev || !slot_off_dev || !blocks_dev) return MOE_EINVAL;
    if (T > 0 && (!rid_dev || !perm_dev || !pos_dev)) return MOE_EINVAL;
    const void *ptrs[] = {rid_dev, act_rep_dev, load_dev, slot_count_dev, slot_off_dev, perm_dev, pos_dev};
    for (const void *p : ptrs)
        if (!moe::aligned(p, 4)) return MOE_EINVAL;
    if (!moe::aligned(blocks_dev, 16)) return MOE_EINVAL;
    a.tb = moe::SchedTables{pl->host_mask_d, pl->slot_of_d, pl->single_rid_d, pl->multi_mask_d, pl->single_mask_d};
    a.n_inst = pl->n_inst; a.C = pl->C; a.n_words = pl->n_words; a.g_self = g_self;
    a.rid = rid_dev; a.act_rep = act_rep_dev; a.load = load_dev;
    a.slot_count = slot_count_dev; a.slot_off = slot_off_dev; a.perm = perm_dev; a.pos = pos_dev; a.blocks = blocks_dev;
    a.block_rows = moe::ffn_block_rows(T);
    a.tail = 1;
    return MOE_OK;
}

}  // namespace

extern "C" int moe_route_schedule_permute(const moe_placement_t *pl, int g_self, const float *logits_dev, int T, int k,
                                          const moe_route_cfg *cfg, int32_t *topk_ids_dev, float *topk_w_dev,
                                          int32_t *rid_dev, int32_t *act_rep_dev, int32_t *load_dev,
                                          int32_t *slot_count_dev, int32_t *slot_off_dev, int32_t *perm_dev,
                                          int32_t *pos_dev, int32_t *blocks_dev, int32_t *sync_dev, void *stream) {
    if (!pl) return MOE_EINVAL;
    const int E = pl->E;
    if (const int rc = check_selection(T, E, k, cfg)) return rc;
    if (!sync_dev || !moe::aligned(sync_dev, 4)) return MOE_EINVAL;
    if (T > 0 && (!logits_dev || !topk_ids_dev || !topk_w_dev)) return MOE_EINVAL;
    if (!moe::aligned(logits_dev, 4) || !moe::aligned(topk_ids_dev, 4) || !moe::aligned(topk_w_dev, 4)) return MOE_EINVAL;
    FrontArgs a{};
    if (const int rc = fill_tail(a, pl, g_self, T, rid_dev, act_rep_dev, load_dev, slot_count_dev, slot_off_dev,
                                 perm_dev, pos_dev, blocks_dev))
        return rc;
    a.logits = logits_dev; a.T = T; a.E = E; a.k = k; a.cfg = *cfg;
    a.ids = topk_ids_dev; a.w = topk_w_dev;
    a.ticket = sync_dev;
    if (T > 0 && front_is_large(pl, T, k)) {
        a.act_bits = reinterpret_cast<uint32_t *>(sync_dev + 1);
        a.hist = sync_dev + 1 + kBitWords;
        a.chunk_pairs = kChunkPairs;
        a.n_chunks = static_cast<int>((static_cast<long long>(T) * k + kChunkPairs - 1) / kChunkPairs);
    }
    return launch_front_for<false>(a, "moe_route_schedule_permute", static_cast<hipStream_t>(stream));
}

extern "C" size_t moe_front_sync_len(const moe_placement_t *pl, int T, int k) {
    if (!pl || T < 0 || k < 1) return 0;
    if (T == 0 || !front_is_large(pl, T, k)) return 1;
    const size_t n_chunks = (static_cast<size_t>(T) * k + kChunkPairs - 1) / kChunkPairs;
    return 1 + kBitWords + n_chunks * pl->C;
}

extern "C" size_t moe_gate_sync_len(int T) { return T > 0 ? 1 + (static_cast<size_t>(T) + 15) / 16 : 1; }

extern "C" int moe_gate_route(const void *X_dev, const void *Wr_dev, const float *bias_dev, int T, int E, int d_h, int k,
                              const moe_route_cfg *cfg, float *logits_dev, int32_t *topk_ids_dev, float *topk_w_dev,
                              int32_t *sync_dev, void *stream) {
    if (const int rc = check_selection(T, E, k, cfg)) return rc;
    if (const int rc = check_gate(X_dev, Wr_dev, bias_dev, logits_dev, T, E, d_h)) return rc;
    if (!sync_dev || !moe::aligned(sync_dev, 4)) return MOE_EINVAL;
    if (T == 0) return MOE_OK;
    if (!topk_ids_dev || !topk_w_dev || !moe::aligned(topk_ids_dev, 4) || !moe::aligned(topk_w_dev, 4)) return MOE_EINVAL;
    FrontArgs a{};
    a.T = T; a.E = E; a.k = k; a.cfg = *cfg;
    a.ids = topk_ids_dev; a.w = topk_w_dev;
    a.ticket = sync_dev;
    a.X = static_cast<const uint16_t *>(X_dev); a.Wr = static_cast<const uint16_t *>(Wr_dev); a.bias = bias_dev;
    a.logits_out = logits_dev; a.d_h = d_h; a.n_tiles = (E + 15) / 16;
    a.n_inst = 1;
    a.tail = 0;
    return launch_front_for<true>(a, "moe_gate_route", static_cast<hipStream_t>(stream));
}

extern "C" int moe_gate_route_schedule_permute(const moe_placement_t *pl, int g_self, const void *X_dev,
                                               const void *Wr_dev, const float *bias_dev, int T, int d_h, int k,
                                               const moe_route_cfg *cfg, float *logits_dev, int32_t *topk_ids_dev,
                                               float *topk_w_dev, int32_t *rid_dev, int32_t *act_rep_dev,
                                               int32_t *load_dev, int32_t *slot_count_dev, int32_t *slot_off_dev,
                                               int32_t *perm_dev, int32_t *pos_dev, int32_t *blocks_dev,
                                               int32_t *sync_dev, void *stream) {
    if (!pl) return MOE_EINVAL;
    const int E = pl->E;
    if (const int rc = check_selection(T, E, k, cfg)) return rc;
    if (const int rc = check_gate(X_dev, Wr_dev, bias_dev, logits_dev, T, E, d_h)) return rc;
    if (!sync_dev || !moe::aligned(sync_dev, 4)) return MOE_EINVAL;
    if (T > 0 && (!topk_ids_dev || !topk_w_dev)) return MOE_EINVAL;
    if (!moe::aligned(topk_ids_dev, 4) || !moe::aligned(topk_w_dev, 4)) return MOE_EINVAL;
    FrontArgs a{};
    if (const int rc = fill_tail(a, pl, g_self, T, rid_dev, act_rep_dev, load_dev, slot_count_dev, slot_off_dev,
                                 perm_dev, pos_dev, blocks_dev))
        return rc;
    a.T = T; a.E = E; a.k = k; a.cfg = *cfg;
    a.ids = topk_ids_dev; a.w = topk_w_dev;
    a.ticket = sync_dev;
    a.X = static_cast<const uint16_t *>(X_dev); a.Wr = static_cast<const uint16_t *>(Wr_dev); a.bias = bias_dev;
    a.logits_out = logits_dev; a.d_h = d_h; a.n_tiles = (E + 15) / 16;
    return launch_front_for<true>(a, "moe_gate_route_schedule_permute", static_cast<hipStream_t>(stream));
}

