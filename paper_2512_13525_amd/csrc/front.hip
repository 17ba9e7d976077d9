// a0-a4 in ONE launch: gating selection for all tokens, then Alg. 1 and this instance's
// dispatch (Janus Sec. 3.4, workflow Steps 0-4).  At decode sizes each of these steps is a few
// microseconds of work behind a launch of about the same cost, so three launches become one.
//
// Every workgroup routes 16 tokens (one per wavefront) and publishes their expert ids with
// agent-scope stores; the workgroup that finishes last (an atomic ticket, nobody waits) then
// runs Alg. 1 and the counting sort on its own, reading the ids with agent-scope loads because
// they were written on other XCDs.
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
};

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

template <int VPL>
__global__ __launch_bounds__(moe::kFrontThreads)
void front_kernel(FrontArgs a) {
    // the phases run one after another, so their LDS overlays
    union Shared {
        float row[moe::kFrontWaves][VPL * MOE_WAVE];
        moe::SchedShared sched;
        moe::PermShared perm;
        SmallShared small;
    };
    __shared__ Shared sh;
    __shared__ int s_last;

    const int wave = threadIdx.x / MOE_WAVE;
    const int lane = moe::lane_id();
    const int t = blockIdx.x * moe::kFrontWaves + wave;
    const int n_pairs = a.T * a.k;
    const bool small = n_pairs <= kRegPairs && a.E * a.n_inst <= kSlotOfLds;
    TablePrefetch tp{};
    if (small) tp = prefetch_tables(a);
    if (t < a.T) {
        moe::route_token<VPL, true>(a.logits + static_cast<size_t>(t) * a.E, a.E, a.k, a.cfg, sh.row[wave], lane,
                                    a.ids + static_cast<size_t>(t) * a.k, a.w + static_cast<size_t>(t) * a.k);
    }
    // a workgroup barrier does not wait for global stores: the ticket must not overtake the ids
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const int old = __hip_atomic_fetch_add(a.ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = old == static_cast<int>(gridDim.x) - 1;
        if (s_last) __hip_atomic_store(a.ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
    }
    __syncthreads();
    if (!s_last) return;

    if (small) {
        front_tail_small(a, sh.small, n_pairs, tp);
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

template <int VPL>
int launch_front(const FrontArgs &a, hipStream_t st) {
    const int blocks = a.T > 0 ? (a.T + moe::kFrontWaves - 1) / moe::kFrontWaves : 1;
    hipLaunchKernelGGL(front_kernel<VPL>, dim3(blocks), dim3(moe::kFrontThreads), 0, st, a);
    return moe::check_launch("moe_route_schedule_permute");
}

}  // namespace

extern "C" int moe_route_schedule_permute(const moe_placement_t *pl, int g_self, const float *logits_dev, int T, int k,
                                          const moe_route_cfg *cfg, int32_t *topk_ids_dev, float *topk_w_dev,
                                          int32_t *rid_dev, int32_t *act_rep_dev, int32_t *load_dev,
                                          int32_t *slot_count_dev, int32_t *slot_off_dev, int32_t *perm_dev,
                                          int32_t *pos_dev, int32_t *blocks_dev, int32_t *sync_dev, void *stream) {
    if (!pl || !cfg || T < 0 || k < 1) return MOE_EINVAL;
    const int E = pl->E;
    if (k > E) return MOE_EINVAL;
    if (k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (static_cast<long long>(T) * k > 0x7fffffffLL) return MOE_ESHAPE;
    if (g_self < 0 || g_self >= pl->n_inst) return MOE_EINVAL;
    if (cfg->mode != MOE_ROUTE_SOFTMAX && cfg->mode != MOE_ROUTE_SIGMOID_GROUP) return MOE_EINVAL;
    if (cfg->mode == MOE_ROUTE_SIGMOID_GROUP) {
        if (cfg->n_group < 1 || cfg->topk_group < 1 || cfg->topk_group > cfg->n_group) return MOE_EINVAL;
        if (cfg->n_group > 64 || E % cfg->n_group != 0 || E / cfg->n_group < 2) return MOE_ESHAPE;
        if (k > cfg->topk_group * (E / cfg->n_group)) return MOE_EINVAL;
    }
    if (!act_rep_dev || !load_dev || !slot_count_dev || !slot_off_dev || !blocks_dev || !sync_dev) return MOE_EINVAL;
    if (T > 0 && (!logits_dev || !topk_ids_dev || !topk_w_dev || !rid_dev || !perm_dev || !pos_dev)) return MOE_EINVAL;
    const void *ptrs[] = {logits_dev, topk_ids_dev, topk_w_dev, rid_dev, act_rep_dev, load_dev,
                          slot_count_dev, slot_off_dev, perm_dev, pos_dev, sync_dev};
    for (const void *p : ptrs)
        if (!moe::aligned(p, 4)) return MOE_EINVAL;
    if (!moe::aligned(blocks_dev, 16)) return MOE_EINVAL;
    FrontArgs a;
    a.logits = logits_dev; a.T = T; a.E = E; a.k = k; a.cfg = *cfg;
    a.ids = topk_ids_dev; a.w = topk_w_dev;
    a.tb = moe::SchedTables{pl->host_mask_d, pl->slot_of_d, pl->single_rid_d, pl->multi_mask_d, pl->single_mask_d};
    a.n_inst = pl->n_inst; a.C = pl->C; a.n_words = pl->n_words; a.g_self = g_self;
    a.rid = rid_dev; a.act_rep = act_rep_dev; a.load = load_dev;
    a.slot_count = slot_count_dev; a.slot_off = slot_off_dev; a.perm = perm_dev; a.pos = pos_dev; a.blocks = blocks_dev;
    a.ticket = sync_dev;
    a.block_rows = moe::ffn_block_rows(T);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int vpl = (E + MOE_WAVE - 1) / MOE_WAVE;
    if (vpl <= 1) return launch_front<1>(a, st);
    if (vpl <= 2) return launch_front<2>(a, st);
    if (vpl <= 4) return launch_front<4>(a, st);
    if (vpl <= 8) return launch_front<8>(a, st);
    return launch_front<16>(a, st);
}
