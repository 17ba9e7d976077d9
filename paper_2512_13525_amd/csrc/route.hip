// a0: gating selection (Janus Sec. 3.4, first step of the scheduling workflow: the gate yields the k
// logical expert ids per token; Sec. 3.3: gating runs on the MoE side over the complete activations).
// One wavefront per token; the selection itself lives in dispatch_dev.h (route_token).
#include "dispatch_dev.h"

namespace {

constexpr int kRouteWavesPerBlock = 4;

// VPL = ceil(E/64) values per lane.
template <int VPL>
__global__ __launch_bounds__(kRouteWavesPerBlock * MOE_WAVE)
void route_kernel(const float *__restrict__ logits, int T, int E, int k, moe_route_cfg cfg,
                  int32_t *__restrict__ topk_ids, float *__restrict__ topk_w) {
    __shared__ float row_lds[kRouteWavesPerBlock][VPL * MOE_WAVE];
    const int wave = threadIdx.x / MOE_WAVE;
    const int lane = moe::lane_id();
    const int t = blockIdx.x * kRouteWavesPerBlock + wave;
    if (t >= T) return;                                  // whole wave leaves; no block barrier is used
    moe::route_token<VPL, false>(logits + static_cast<size_t>(t) * E, E, k, cfg, row_lds[wave], lane,
                                 topk_ids + static_cast<size_t>(t) * k, topk_w + static_cast<size_t>(t) * k);
}

template <int VPL>
int launch_route(const float *logits, int T, int E, int k, const moe_route_cfg &cfg,
                 int32_t *ids, float *w, hipStream_t st) {
    const int blocks = (T + kRouteWavesPerBlock - 1) / kRouteWavesPerBlock;
    hipLaunchKernelGGL(route_kernel<VPL>, dim3(blocks), dim3(kRouteWavesPerBlock * MOE_WAVE), 0, st,
                       logits, T, E, k, cfg, ids, w);
    return moe::check_launch("moe_route");
}

}  // namespace

extern "C" int moe_route(const float *logits_dev, int T, int E, int k, const moe_route_cfg *cfg,
                         int32_t *topk_ids_dev, float *topk_w_dev, void *stream) {
    if (!cfg) return MOE_EINVAL;
    if (T < 0 || E < 1 || k < 1 || k > E) return MOE_EINVAL;
    if (E > MOE_MAX_EXPERTS || k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (cfg->mode != MOE_ROUTE_SOFTMAX && cfg->mode != MOE_ROUTE_SIGMOID_GROUP) return MOE_EINVAL;
    if (cfg->mode == MOE_ROUTE_SIGMOID_GROUP) {
        if (cfg->n_group < 1 || cfg->topk_group < 1 || cfg->topk_group > cfg->n_group) return MOE_EINVAL;
        if (cfg->n_group > 64 || E % cfg->n_group != 0 || E / cfg->n_group < 2) return MOE_ESHAPE;
        if (k > cfg->topk_group * (E / cfg->n_group)) return MOE_EINVAL;
    }
    if (T == 0) return MOE_OK;
    if (!logits_dev || !topk_ids_dev || !topk_w_dev) return MOE_EINVAL;
    if (!moe::aligned(logits_dev, 4) || !moe::aligned(topk_ids_dev, 4) || !moe::aligned(topk_w_dev, 4))
        return MOE_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int vpl = (E + MOE_WAVE - 1) / MOE_WAVE;
    if (vpl <= 1) return launch_route<1>(logits_dev, T, E, k, *cfg, topk_ids_dev, topk_w_dev, st);
    if (vpl <= 2) return launch_route<2>(logits_dev, T, E, k, *cfg, topk_ids_dev, topk_w_dev, st);
    if (vpl <= 4) return launch_route<4>(logits_dev, T, E, k, *cfg, topk_ids_dev, topk_w_dev, st);
    if (vpl <= 8) return launch_route<8>(logits_dev, T, E, k, *cfg, topk_ids_dev, topk_w_dev, st);
    return launch_route<16>(logits_dev, T, E, k, *cfg, topk_ids_dev, topk_w_dev, st);
}
