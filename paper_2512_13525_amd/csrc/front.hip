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
    int32_t *rid, *act_rep, *load, *slot_count, *slot_off, *perm, *pos;
    int32_t *ticket;
};

template <int VPL>
__global__ __launch_bounds__(moe::kFrontThreads)
void front_kernel(FrontArgs a) {
    // the phases run one after another, so their LDS overlays
    union Shared {
        float row[moe::kFrontWaves][VPL * MOE_WAVE];
        moe::SchedShared sched;
        moe::PermShared perm;
    };
    __shared__ Shared sh;
    __shared__ int s_last;

    const int wave = threadIdx.x / MOE_WAVE;
    const int lane = moe::lane_id();
    const int t = blockIdx.x * moe::kFrontWaves + wave;
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

    const int n_pairs = a.T * a.k;
    const int vec_ok = ((reinterpret_cast<uintptr_t>(a.ids) | reinterpret_cast<uintptr_t>(a.rid)) & 15) == 0;
    moe::aebs_block(a.tb, sh.sched, a.E, a.n_inst, a.C, a.n_words, a.ids, n_pairs, vec_ok, true,
                    a.rid, a.act_rep, a.load);
    // rid is re-read below by other wavefronts of this workgroup
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    moe::permute_block(sh.perm, a.rid, n_pairs, a.g_self, a.C, a.slot_count, a.slot_off, a.perm, a.pos);
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
                                          int32_t *pos_dev, int32_t *sync_dev, void *stream) {
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
    if (!act_rep_dev || !load_dev || !slot_count_dev || !slot_off_dev || !sync_dev) return MOE_EINVAL;
    if (T > 0 && (!logits_dev || !topk_ids_dev || !topk_w_dev || !rid_dev || !perm_dev || !pos_dev)) return MOE_EINVAL;
    const void *ptrs[] = {logits_dev, topk_ids_dev, topk_w_dev, rid_dev, act_rep_dev, load_dev,
                          slot_count_dev, slot_off_dev, perm_dev, pos_dev, sync_dev};
    for (const void *p : ptrs)
        if (!moe::aligned(p, 4)) return MOE_EINVAL;
    FrontArgs a;
    a.logits = logits_dev; a.T = T; a.E = E; a.k = k; a.cfg = *cfg;
    a.ids = topk_ids_dev; a.w = topk_w_dev;
    a.tb = moe::SchedTables{pl->host_mask_d, pl->slot_of_d, pl->single_rid_d, pl->multi_mask_d, pl->single_mask_d};
    a.n_inst = pl->n_inst; a.C = pl->C; a.n_words = pl->n_words; a.g_self = g_self;
    a.rid = rid_dev; a.act_rep = act_rep_dev; a.load = load_dev;
    a.slot_count = slot_count_dev; a.slot_off = slot_off_dev; a.perm = perm_dev; a.pos = pos_dev;
    a.ticket = sync_dev;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int vpl = (E + MOE_WAVE - 1) / MOE_WAVE;
    if (vpl <= 1) return launch_front<1>(a, st);
    if (vpl <= 2) return launch_front<2>(a, st);
    if (vpl <= 4) return launch_front<4>(a, st);
    if (vpl <= 8) return launch_front<8>(a, st);
    return launch_front<16>(a, st);
}
