// a4: this instance's share of the dispatch (Janus Sec. 3.4, Step 4) and
// a6: the weighted top-k combine that produces the instance-partial output entering the
// reverse-path reduction (Sec. 3.3).
//
// permute: a stable counting sort of the local requests by slot, one workgroup of 16
// wavefronts.  Each wavefront owns a contiguous range of request ids, so "ascending request
// id inside a slot" follows from (wave order, group order, lane order) and never from the
// arrival order of atomics:
//   pass A  per-(wave, slot) histograms in LDS;
//   scan    per-slot exclusive prefix over waves, then an exclusive scan over slots;
//   pass B  each wave walks its range again; the lanes of a 64-request group that share a
//           slot are found with a ballot, ranked with a popcount of the lower lanes, and
//           written at the wave's running base for that slot.
#include "common.h"

namespace {

constexpr int kPermThreads = 1024;
constexpr int kPermWaves = kPermThreads / MOE_WAVE;

__global__ __launch_bounds__(kPermThreads)
void permute_kernel(const int32_t *__restrict__ rid, int n_pairs, int g_self, int C,
                    int32_t *__restrict__ slot_count, int32_t *__restrict__ slot_off,
                    int32_t *__restrict__ perm, int32_t *__restrict__ pos) {
    __shared__ int cnt[kPermWaves][MOE_MAX_SLOTS];     // pass A: counts; pass B: running bases
    __shared__ int total[MOE_MAX_SLOTS];
    __shared__ int off_lds[MOE_MAX_SLOTS + 1];

    const int tid = threadIdx.x;
    const int wave = tid / MOE_WAVE;
    const int lane = tid % MOE_WAVE;
    for (int i = tid; i < kPermWaves * MOE_MAX_SLOTS; i += kPermThreads) (&cnt[0][0])[i] = 0;
    __syncthreads();

    const int n_groups = (n_pairs + MOE_WAVE - 1) / MOE_WAVE;
    const int gpw = (n_groups + kPermWaves - 1) / kPermWaves;
    const int g_begin = wave * gpw;
    const int g_end = min(n_groups, g_begin + gpw);
    const int rid_lo = g_self * C;

    // ---- pass A
    for (int grp = g_begin; grp < g_end; ++grp) {
        const int p = grp * MOE_WAVE + lane;
        const int s = (p < n_pairs ? rid[p] : -1) - rid_lo;
        if (p < n_pairs && s >= 0 && s < C) atomicAdd(&cnt[wave][s], 1);
    }
    __syncthreads();

    // ---- per-slot exclusive prefix over waves
    for (int s = tid; s < C; s += kPermThreads) {
        int run = 0;
#pragma unroll
        for (int w = 0; w < kPermWaves; ++w) {
            const int c = cnt[w][s];
            cnt[w][s] = run;
            run += c;
        }
        total[s] = run;
        slot_count[s] = run;
    }
    __syncthreads();

    // ---- exclusive scan over slots (first wavefront, 64 slots per round)
    if (wave == 0) {
        int carry = 0;
        for (int s0 = 0; s0 < C; s0 += MOE_WAVE) {
            const int s = s0 + lane;
            const int v = s < C ? total[s] : 0;
            int incl = v;
#pragma unroll
            for (int d = 1; d < MOE_WAVE; d <<= 1) {
                const int o = __shfl_up(incl, d, MOE_WAVE);
                if (lane >= d) incl += o;
            }
            if (s < C) {
                off_lds[s] = carry + incl - v;
                slot_off[s] = carry + incl - v;
            }
            carry += __shfl(incl, MOE_WAVE - 1, MOE_WAVE);
        }
        if (lane == 0) {
            off_lds[C] = carry;
            slot_off[C] = carry;
        }
    }
    __syncthreads();

    // ---- pass B
    volatile int *base = &cnt[wave][0];
    for (int grp = g_begin; grp < g_end; ++grp) {
        const int p = grp * MOE_WAVE + lane;
        const int s = (p < n_pairs ? rid[p] : -1) - rid_lo;
        const bool local = p < n_pairs && s >= 0 && s < C;
        int row = -1;
        uint64_t todo = __ballot(local);
        while (todo) {
            const int lead = __builtin_ctzll(todo);
            const int s0 = __builtin_amdgcn_readlane(s, lead);
            const uint64_t same = __ballot(local && s == s0);
            const int b = base[s0] + off_lds[s0];
            if (local && s == s0) row = b + __popcll(same & moe::lanemask_lt());
            __builtin_amdgcn_wave_barrier();
            if (lane == lead) base[s0] += __popcll(same);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            todo &= ~same;
        }
        if (p < n_pairs) {
            pos[p] = row;
            if (local) perm[row] = p;
        }
    }
}

// One workgroup per (token, 1024-column chunk); each thread owns 4 consecutive columns.
template <bool OUT_BF16>
__global__ __launch_bounds__(256)
void combine_kernel(const float *__restrict__ Yp, const int32_t *__restrict__ pos,
                    const float *__restrict__ w, int k, int d_h, void *__restrict__ Y) {
    const int i = blockIdx.x;
    const int col = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (col >= d_h) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < k; ++j) {
        const int r = pos[i * k + j];
        if (r < 0) continue;
        const float wj = w[i * k + j];
        const float4 y = *reinterpret_cast<const float4 *>(Yp + static_cast<size_t>(r) * d_h + col);
        acc.x += wj * y.x; acc.y += wj * y.y; acc.z += wj * y.z; acc.w += wj * y.w;
    }
    if (OUT_BF16) {
        ushort4 o;
        o.x = moe::f32_to_bf16(acc.x); o.y = moe::f32_to_bf16(acc.y);
        o.z = moe::f32_to_bf16(acc.z); o.w = moe::f32_to_bf16(acc.w);
        *reinterpret_cast<ushort4 *>(static_cast<uint16_t *>(Y) + static_cast<size_t>(i) * d_h + col) = o;
    } else {
        *reinterpret_cast<float4 *>(static_cast<float *>(Y) + static_cast<size_t>(i) * d_h + col) = acc;
    }
}

}  // namespace

extern "C" int moe_permute(const moe_placement_t *pl, int g_self, const int32_t *rid_dev, int T, int k,
                           int32_t *slot_count_dev, int32_t *slot_off_dev, int32_t *perm_dev,
                           int32_t *pos_dev, void *stream) {
    if (!pl || T < 0 || k < 1) return MOE_EINVAL;
    if (g_self < 0 || g_self >= pl->n_inst) return MOE_EINVAL;
    if (k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (static_cast<long long>(T) * k > 0x7fffffffLL) return MOE_ESHAPE;
    if (!slot_count_dev || !slot_off_dev) return MOE_EINVAL;
    if (T > 0 && (!rid_dev || !perm_dev || !pos_dev)) return MOE_EINVAL;
    if (!moe::aligned(rid_dev, 4) || !moe::aligned(slot_count_dev, 4) || !moe::aligned(slot_off_dev, 4) ||
        !moe::aligned(perm_dev, 4) || !moe::aligned(pos_dev, 4))
        return MOE_EINVAL;
    hipLaunchKernelGGL(permute_kernel, dim3(1), dim3(kPermThreads), 0, static_cast<hipStream_t>(stream),
                       rid_dev, T * k, g_self, pl->C, slot_count_dev, slot_off_dev, perm_dev, pos_dev);
    return moe::check_launch("moe_permute");
}

extern "C" int moe_combine(const float *Yp_dev, const int32_t *pos_dev, const float *topk_w_dev,
                           int T, int k, int d_h, int dtype, void *Y_dev, void *stream) {
    if (T < 0 || k < 1 || d_h < 1) return MOE_EINVAL;
    if (dtype != MOE_DTYPE_BF16 && dtype != MOE_DTYPE_F32) return MOE_EINVAL;
    if (d_h % 4 != 0 || k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (T == 0) return MOE_OK;
    if (!Yp_dev || !pos_dev || !topk_w_dev || !Y_dev) return MOE_EINVAL;
    if (!moe::aligned(Yp_dev, 16) || !moe::aligned(pos_dev, 4) || !moe::aligned(topk_w_dev, 4) ||
        !moe::aligned(Y_dev, dtype == MOE_DTYPE_BF16 ? 8 : 16))
        return MOE_EINVAL;
    const dim3 grid(T, (d_h + 1023) / 1024);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == MOE_DTYPE_BF16)
        hipLaunchKernelGGL(combine_kernel<true>, grid, dim3(256), 0, st, Yp_dev, pos_dev, topk_w_dev, k, d_h, Y_dev);
    else
        hipLaunchKernelGGL(combine_kernel<false>, grid, dim3(256), 0, st, Yp_dev, pos_dev, topk_w_dev, k, d_h, Y_dev);
    return moe::check_launch("moe_combine");
}
