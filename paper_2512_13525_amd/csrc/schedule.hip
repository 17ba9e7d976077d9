// a1-a3: Activated-Expert-Balanced Scheduling (Janus Sec. 3.4, Alg. 1) as one kernel of one
// workgroup; the algorithm itself lives in dispatch_dev.h (aebs_block).
#include "dispatch_dev.h"

namespace {

using moe::SchedTables;
constexpr int kSchedThreads = moe::kFrontThreads;

// One workgroup per batch (blockIdx.x): batch b reads ids + b*n_pairs and writes rid + b*n_pairs,
// act_rep + b*E, load_out + b*n_inst.  The single-batch call is a grid of one.
__global__ __launch_bounds__(kSchedThreads)
void aebs_kernel(SchedTables tb, int E, int n_inst, int C, int n_words,
                 const int32_t *__restrict__ ids, int n_pairs, int vec_ok,
                 int32_t *__restrict__ rid, int32_t *__restrict__ act_rep, int32_t *__restrict__ load_out) {
    __shared__ moe::SchedShared sh;
    const size_t b = blockIdx.x;
    moe::aebs_block(tb, sh, E, n_inst, C, n_words, ids + b * n_pairs, n_pairs, vec_ok, false,
                    rid ? rid + b * n_pairs : nullptr, act_rep ? act_rep + b * E : nullptr, load_out + b * n_inst);
}

// Baseline policies the paper compares AEBS with (Sec. 5): every request of expert e goes to e's
// first replica (MOE_POLICY_HOME: no scheduling), or to replica number draw mod R(e) of e, replicas
// in ascending instance order (MOE_POLICY_RANDOM: balances tokens, not activated experts).  One
// workgroup; load[g] = distinct replicas of instance g that received a request, counted through a
// bitset of all n_inst*C replica ids in LDS.
__global__ __launch_bounds__(kSchedThreads)
void baseline_kernel(const uint64_t *__restrict__ host_mask, const int16_t *__restrict__ slot_of, int n_inst, int C,
                     const int32_t *__restrict__ ids, const uint32_t *__restrict__ draws, int n_pairs, int policy,
                     int32_t *__restrict__ rid, int32_t *__restrict__ load_out) {
    __shared__ uint32_t used[MOE_MAX_INSTANCES * MOE_MAX_SLOTS / 32];
    __shared__ int load[MOE_MAX_INSTANCES];
    const int n_rids = n_inst * C;
    // one workgroup per batch
    ids += static_cast<size_t>(blockIdx.x) * n_pairs;
    if (draws) draws += static_cast<size_t>(blockIdx.x) * n_pairs;
    if (rid) rid += static_cast<size_t>(blockIdx.x) * n_pairs;
    load_out += static_cast<size_t>(blockIdx.x) * n_inst;
    for (int i = threadIdx.x; i < (n_rids + 31) / 32; i += kSchedThreads) used[i] = 0u;
    if (threadIdx.x < n_inst) load[threadIdx.x] = 0;
    __syncthreads();
    for (int p = threadIdx.x; p < n_pairs; p += kSchedThreads) {
        const int e = ids[p];
        uint64_t hosts = host_mask[e];
        int skip = policy == MOE_POLICY_RANDOM ? static_cast<int>(draws[p] % static_cast<uint32_t>(__popcll(hosts))) : 0;
        while (skip-- > 0) hosts &= hosts - 1;                   // drop the lowest instances
        const int g = __builtin_ctzll(hosts);
        const int r = g * C + slot_of[e * n_inst + g];
        if (rid) rid[p] = r;
        atomicOr(&used[r >> 5], 1u << (r & 31));
    }
    __syncthreads();
    for (int r = threadIdx.x; r < n_rids; r += kSchedThreads)
        if ((used[r >> 5] >> (r & 31)) & 1u) atomicAdd(&load[r / C], 1);
    __syncthreads();
    if (threadIdx.x < n_inst) load_out[threadIdx.x] = load[threadIdx.x];
}

}  // namespace

extern "C" int moe_schedule_baseline(const moe_placement_t *pl, const int32_t *topk_ids_dev, int T, int k,
                                     int policy, const uint32_t *draws_dev, int32_t *rid_dev, int32_t *load_dev,
                                     void *stream) {
    if (!pl || T < 0 || k < 1) return MOE_EINVAL;
    if (policy != MOE_POLICY_HOME && policy != MOE_POLICY_RANDOM) return MOE_EINVAL;
    if (k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (static_cast<long long>(T) * k > 0x7fffffffLL) return MOE_ESHAPE;
    if (!load_dev) return MOE_EINVAL;
    if (T > 0 && (!topk_ids_dev || !rid_dev || (policy == MOE_POLICY_RANDOM && !draws_dev))) return MOE_EINVAL;
    if (!moe::aligned(topk_ids_dev, 4) || !moe::aligned(rid_dev, 4) || !moe::aligned(draws_dev, 4) ||
        !moe::aligned(load_dev, 4))
        return MOE_EINVAL;
    hipLaunchKernelGGL(baseline_kernel, dim3(1), dim3(kSchedThreads), 0, static_cast<hipStream_t>(stream),
                       pl->host_mask_d, pl->slot_of_d, pl->n_inst, pl->C, topk_ids_dev, draws_dev, T * k, policy,
                       rid_dev, load_dev);
    return moe::check_launch("moe_schedule_baseline");
}

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

// The batched forms for the Monte-Carlo estimate of a_max(n_e, B) (Sec. 3.5: the table Alg. 2 reads is built
// by sampling batches and scheduling them): one launch, one workgroup per sampled batch.
extern "C" int moe_schedule_batched(const moe_placement_t *pl, const int32_t *topk_ids_dev, int n_batches, int T, int k,
                                    int32_t *rid_dev, int32_t *act_rep_dev, int32_t *load_dev, void *stream) {
    if (!pl || n_batches < 0 || T < 0 || k < 1) return MOE_EINVAL;
    if (k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (static_cast<long long>(T) * k > 0x7fffffffLL || n_batches > 0x7fffffff / 2) return MOE_ESHAPE;
    if (n_batches == 0) return MOE_OK;
    if (!load_dev || (T > 0 && !topk_ids_dev)) return MOE_EINVAL;
    if (!moe::aligned(topk_ids_dev, 4) || !moe::aligned(rid_dev, 4) || !moe::aligned(act_rep_dev, 4) ||
        !moe::aligned(load_dev, 4))
        return MOE_EINVAL;
    // 16-byte accesses need every batch's rows aligned, not only the first
    const int vec_ok = moe::aligned(topk_ids_dev, 16) && (!rid_dev || moe::aligned(rid_dev, 16)) &&
                       (static_cast<long long>(T) * k) % 4 == 0;
    SchedTables tb{pl->host_mask_d, pl->slot_of_d, pl->single_rid_d, pl->multi_mask_d, pl->single_mask_d};
    hipLaunchKernelGGL(aebs_kernel, dim3(n_batches), dim3(kSchedThreads), 0, static_cast<hipStream_t>(stream),
                       tb, pl->E, pl->n_inst, pl->C, pl->n_words, topk_ids_dev, T * k, vec_ok,
                       rid_dev, act_rep_dev, load_dev);
    return moe::check_launch("moe_schedule_batched");
}

extern "C" int moe_schedule_baseline_batched(const moe_placement_t *pl, const int32_t *topk_ids_dev, int n_batches, int T,
                                             int k, int policy, const uint32_t *draws_dev, int32_t *rid_dev,
                                             int32_t *load_dev, void *stream) {
    if (!pl || n_batches < 0 || T < 0 || k < 1) return MOE_EINVAL;
    if (policy != MOE_POLICY_HOME && policy != MOE_POLICY_RANDOM) return MOE_EINVAL;
    if (k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (static_cast<long long>(T) * k > 0x7fffffffLL || n_batches > 0x7fffffff / 2) return MOE_ESHAPE;
    if (n_batches == 0) return MOE_OK;
    if (!load_dev) return MOE_EINVAL;
    if (T > 0 && (!topk_ids_dev || (policy == MOE_POLICY_RANDOM && !draws_dev))) return MOE_EINVAL;
    if (!moe::aligned(topk_ids_dev, 4) || !moe::aligned(rid_dev, 4) || !moe::aligned(draws_dev, 4) ||
        !moe::aligned(load_dev, 4))
        return MOE_EINVAL;
    hipLaunchKernelGGL(baseline_kernel, dim3(n_batches), dim3(kSchedThreads), 0, static_cast<hipStream_t>(stream),
                       pl->host_mask_d, pl->slot_of_d, pl->n_inst, pl->C, topk_ids_dev,
                       policy == MOE_POLICY_RANDOM ? draws_dev : nullptr, T * k, policy, rid_dev, load_dev);
    return moe::check_launch("moe_schedule_baseline_batched");
}
