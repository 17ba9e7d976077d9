// a1-a3: Activated-Expert-Balanced Scheduling (Janus Sec. 3.4, Alg. 1) as one kernel of one
// workgroup; the algorithm itself lives in dispatch_dev.h (aebs_block).
#include "dispatch_dev.h"

namespace {

using moe::SchedTables;
constexpr int kSchedThreads = moe::kFrontThreads;

__global__ __launch_bounds__(kSchedThreads)
void aebs_kernel(SchedTables tb, int E, int n_inst, int C, int n_words,
                 const int32_t *__restrict__ ids, int n_pairs, int vec_ok,
                 int32_t *__restrict__ rid, int32_t *__restrict__ act_rep, int32_t *__restrict__ load_out) {
    __shared__ moe::SchedShared sh;
    moe::aebs_block(tb, sh, E, n_inst, C, n_words, ids, n_pairs, vec_ok, false, rid, act_rep, load_out);
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
