// a0: gating selection (Janus Sec. 3.4 workflow: "gating first produces the top-k logical
// expert ids"; Sec. 3.3: gating runs on the MoE side over the complete activations).
//
// One wavefront per token.  Lane l owns experts l, l+64, l+128, ...; every logit is turned
// into a 64-bit key (order-preserving float bits in the high word, ~id in the low word) so
// that "largest logit, lower id on ties" is a plain unsigned maximum, found with a 6-step
// cross-lane butterfly.  The k selections are k such reductions; the winner's key is
// cleared in the owning lane.
#include "common.h"

namespace {

constexpr int kRouteWavesPerBlock = 4;

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        uint64_t o = __shfl_xor(v, off, MOE_WAVE);
        v = o > v ? o : v;
    }
    return v;
}

__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, MOE_WAVE);
    return v;
}

__device__ __forceinline__ uint32_t orderable(float f) {
    uint32_t u = __float_as_uint(f + 0.0f);            // -0.0 -> +0.0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float from_orderable(uint32_t o) {
    uint32_t u = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
    return __uint_as_float(u);
}

__device__ __forceinline__ uint64_t make_key(float v, int id) {
    return (static_cast<uint64_t>(orderable(v)) << 32) | static_cast<uint32_t>(0x7fffffff - id);
}

__device__ __forceinline__ float sigmoid_f32(float x) { return 1.0f / (1.0f + expf(-x)); }

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
    const float *row = logits + static_cast<size_t>(t) * E;

    float v[VPL];
    uint64_t key[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int e = lane + i * MOE_WAVE;
        v[i] = e < E ? row[e] : 0.0f;
        key[i] = e < E ? make_key(v[i], e) : 0ull;
    }

    float denom_all = 0.0f;                              // softmax denominator over all experts
    if (cfg.mode == MOE_ROUTE_SIGMOID_GROUP) {
        // group score = sum of the two largest sigmoid scores of the group, in fp32
        const int per = E / cfg.n_group;
#pragma unroll
        for (int i = 0; i < VPL; ++i) row_lds[wave][lane + i * MOE_WAVE] = v[i];
        // the row is private to this wave: a wavefront-scope fence orders its LDS writes
        // before the reads below (no block barrier: waves past T have already left)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint64_t gkey = 0ull;
        if (lane < cfg.n_group) {
            float a = -INFINITY, b = -INFINITY;          // a >= b: two largest logits of the group
            for (int j = 0; j < per; ++j) {
                const float x = row_lds[wave][lane * per + j];
                if (x > a) { b = a; a = x; }
                else if (x > b) { b = x; }
            }
            const float score = sigmoid_f32(a) + sigmoid_f32(b);
            gkey = make_key(score, lane);
        }
        uint64_t keep = 0ull;
        for (int j = 0; j < cfg.topk_group; ++j) {
            const uint64_t best = wave_max_u64(gkey);
            const int g = 0x7fffffff - static_cast<int>(best & 0xffffffffu);
            keep |= 1ull << g;
            if (lane == g) gkey = 0ull;
        }
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int e = lane + i * MOE_WAVE;
            if (e < E && !((keep >> (e / per)) & 1ull)) key[i] = 0ull;
        }
    } else if (!cfg.renormalize) {
        uint64_t m = 0ull;
#pragma unroll
        for (int i = 0; i < VPL; ++i) m = key[i] > m ? key[i] : m;
        const float vmax = from_orderable(static_cast<uint32_t>(wave_max_u64(m) >> 32));
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < VPL; ++i)
            if (lane + i * MOE_WAVE < E) s += expf(v[i] - vmax);
        denom_all = wave_sum_f32(s);
    }

    // k rounds of "largest remaining"
    float sel_v = 0.0f;            // lane j keeps the j-th selected logit
    int sel_id = 0;
    float vmax = 0.0f;
    for (int j = 0; j < k; ++j) {
        uint64_t m = 0ull;
#pragma unroll
        for (int i = 0; i < VPL; ++i) m = key[i] > m ? key[i] : m;
        const uint64_t best = wave_max_u64(m);
        const int id = 0x7fffffff - static_cast<int>(best & 0xffffffffu);
        const float val = from_orderable(static_cast<uint32_t>(best >> 32));
        if (j == 0) vmax = val;
        if (lane == j) { sel_v = val; sel_id = id; }
#pragma unroll
        for (int i = 0; i < VPL; ++i)
            if (lane + i * MOE_WAVE == id) key[i] = 0ull;
    }

    // weights of the k selected experts (lanes 0..k-1)
    float score = 0.0f;
    if (lane < k) {
        score = cfg.mode == MOE_ROUTE_SIGMOID_GROUP ? sigmoid_f32(sel_v) : expf(sel_v - vmax);
    }
    const float denom_sel = wave_sum_f32(score);
    if (lane < k) {
        float w;
        if (cfg.mode == MOE_ROUTE_SIGMOID_GROUP) w = score / denom_sel * cfg.scale;
        else if (cfg.renormalize) w = score / denom_sel;
        else w = score / denom_all;
        topk_ids[static_cast<size_t>(t) * k + lane] = sel_id;
        topk_w[static_cast<size_t>(t) * k + lane] = w;
    }
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
