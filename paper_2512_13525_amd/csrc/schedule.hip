// a1-a3: Activated-Expert-Balanced Scheduling (Janus Sec. 3.4, Alg. 1) as one kernel.
//
// One workgroup of 16 wavefronts runs the whole algorithm, so the three steps need no
// grid-wide synchronisation and the schedule is a pure function of (layout, activated set):
//   Step 1 (collect)  every thread scans a strided share of the request ids and raises a
//                     flag per expert in LDS (all writers store the same value);
//   Step 2 (select)   one wavefront turns the flags into 64-bit ballots.  Loads of
//                     single-replica experts are popcounts of (ballot & per-instance mask);
//                     lane g holds load[g] in a register.  Multi-replica experts are walked
//                     in ascending id by peeling bits off (ballot & multi-replica mask); the
//                     arg-min over the expert's hosts reads the candidate lanes' loads with
//                     scalar-indexed lane reads, so one greedy step costs a few scalar
//                     instructions per host;
//   Step 3 (rewrite)  every thread maps its share of requests through actRep held in LDS.
// The layout tables are staged into LDS while Step 1 runs.
#include "common.h"

namespace {

constexpr int kSchedThreads = 1024;

struct SchedTables {
    const uint64_t *host_mask;     // [E]
    const int16_t  *slot_of;       // [E*n_inst]
    const int32_t  *single_rid;    // [E]
    const uint64_t *multi_mask;    // [n_words]
    const uint64_t *single_mask;   // [n_inst*n_words]
};

__device__ __forceinline__ uint64_t readlane_u64(uint64_t v, int l) {
    const uint32_t lo = __builtin_amdgcn_readlane(static_cast<int>(v & 0xffffffffu), l);
    const uint32_t hi = __builtin_amdgcn_readlane(static_cast<int>(v >> 32), l);
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

__device__ __forceinline__ uint64_t readfirstlane_u64(uint64_t v) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<int>(v & 0xffffffffu));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<int>(v >> 32));
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

__global__ __launch_bounds__(kSchedThreads)
void aebs_kernel(SchedTables tb, int E, int n_inst, int C, int n_words,
                 const int32_t *__restrict__ ids, int n_pairs, int vec_ok,
                 int32_t *__restrict__ rid, int32_t *__restrict__ act_rep, int32_t *__restrict__ load_out) {
    __shared__ uint32_t flag[MOE_MAX_EXPERTS];
    __shared__ int32_t rep_lds[MOE_MAX_EXPERTS];
    __shared__ uint64_t host_mask_lds[MOE_MAX_EXPERTS];
    __shared__ int32_t single_rid_lds[MOE_MAX_EXPERTS];
    __shared__ uint64_t multi_mask_lds[MOE_MAX_EXPERTS / 64];
    __shared__ uint64_t single_mask_lds[MOE_MAX_INSTANCES * (MOE_MAX_EXPERTS / 64)];

    const int tid = threadIdx.x;
    for (int e = tid; e < E; e += kSchedThreads) {
        flag[e] = 0u;
        host_mask_lds[e] = tb.host_mask[e];
        single_rid_lds[e] = tb.single_rid[e];
    }
    for (int i = tid; i < n_words; i += kSchedThreads) multi_mask_lds[i] = tb.multi_mask[i];
    for (int i = tid; i < n_inst * n_words; i += kSchedThreads) single_mask_lds[i] = tb.single_mask[i];
    __syncthreads();

    // ---- Step 1: collect the activated experts
    if (vec_ok) {
        const int n4 = n_pairs >> 2;
        const int4 *ids4 = reinterpret_cast<const int4 *>(ids);
        for (int i = tid; i < n4; i += kSchedThreads) {
            const int4 v = ids4[i];
            flag[v.x] = 1u; flag[v.y] = 1u; flag[v.z] = 1u; flag[v.w] = 1u;
        }
        for (int i = (n4 << 2) + tid; i < n_pairs; i += kSchedThreads) flag[ids[i]] = 1u;
    } else {
        for (int i = tid; i < n_pairs; i += kSchedThreads) flag[ids[i]] = 1u;
    }
    __syncthreads();

    // ---- Step 2: select one replica per activated expert (first wavefront)
    if (tid < MOE_WAVE) {
        const int lane = tid;
        int load = 0;                                   // lane g: load[g]
        for (int w = 0; w < n_words; ++w) {
            const int e = w * 64 + lane;
            const uint64_t act = __ballot(e < E && flag[e] != 0u);
            if (lane < n_inst) load += __popcll(act & single_mask_lds[lane * n_words + w]);
        }
        for (int w = 0; w < n_words; ++w) {
            const int e = w * 64 + lane;
            const uint64_t act = __ballot(e < E && flag[e] != 0u);
            const uint64_t hm = e < E ? host_mask_lds[e] : 0ull;
            uint64_t todo = act & readfirstlane_u64(multi_mask_lds[w]);   // wave-uniform: keep the loop scalar
            int chosen = -1;                            // lane b: instance chosen for expert w*64+b
            while (todo) {
                const int b = __builtin_ctzll(todo);
                todo &= todo - 1;
                uint64_t hosts = readlane_u64(hm, b);
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
                    if (chosen >= 0) rep = chosen * C + tb.slot_of[e * n_inst + chosen];
                    else rep = single_rid_lds[e];
                }
                rep_lds[e] = rep;
                act_rep[e] = rep;
            }
        }
        if (lane < n_inst) load_out[lane] = load;
    }
    __syncthreads();

    // ---- Step 3: rewrite every request
    if (vec_ok) {
        const int n4 = n_pairs >> 2;
        const int4 *ids4 = reinterpret_cast<const int4 *>(ids);
        int4 *rid4 = reinterpret_cast<int4 *>(rid);
        for (int i = tid; i < n4; i += kSchedThreads) {
            const int4 v = ids4[i];
            int4 r;
            r.x = rep_lds[v.x]; r.y = rep_lds[v.y]; r.z = rep_lds[v.z]; r.w = rep_lds[v.w];
            rid4[i] = r;
        }
        for (int i = (n4 << 2) + tid; i < n_pairs; i += kSchedThreads) rid[i] = rep_lds[ids[i]];
    } else {
        for (int i = tid; i < n_pairs; i += kSchedThreads) rid[i] = rep_lds[ids[i]];
    }
}

}  // namespace

extern "C" int moe_schedule(const moe_placement_t *pl, const int32_t *topk_ids_dev, int T, int k,
                            int32_t *rid_dev, int32_t *act_rep_dev, int32_t *load_dev, void *stream) {
    if (!pl || T < 0 || k < 1) return MOE_EINVAL;
    if (k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (static_cast<long long>(T) * k > 0x7fffffffLL) return MOE_ESHAPE;
    if (!act_rep_dev || !load_dev) return MOE_EINVAL;
    if (T > 0 && (!topk_ids_dev || !rid_dev)) return MOE_EINVAL;
    if (!moe::aligned(topk_ids_dev, 4) || !moe::aligned(rid_dev, 4) || !moe::aligned(act_rep_dev, 4) ||
        !moe::aligned(load_dev, 4))
        return MOE_EINVAL;
    const int vec_ok = moe::aligned(topk_ids_dev, 16) && moe::aligned(rid_dev, 16);
    SchedTables tb{pl->host_mask_d, pl->slot_of_d, pl->single_rid_d, pl->multi_mask_d, pl->single_mask_d};
    hipLaunchKernelGGL(aebs_kernel, dim3(1), dim3(kSchedThreads), 0, static_cast<hipStream_t>(stream),
                       tb, pl->E, pl->n_inst, pl->C, pl->n_words, topk_ids_dev, T * k, vec_ok,
                       rid_dev, act_rep_dev, load_dev);
    return moe::check_launch("moe_schedule");
}
