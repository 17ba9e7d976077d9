// a4: this instance's share of the dispatch (Janus Sec. 3.4, Step 4) and
// a6: the weighted top-k combine that produces the instance-partial output entering the
// reverse-path reduction (Sec. 3.3).  The counting sort lives in dispatch_dev.h (permute_block).
#include "dispatch_dev.h"

namespace {

constexpr int kPermThreads = moe::kFrontThreads;

__global__ __launch_bounds__(kPermThreads)
void permute_kernel(const int32_t *__restrict__ rid, int n_pairs, int g_self, int C,
                    int32_t *__restrict__ slot_count, int32_t *__restrict__ slot_off,
                    int32_t *__restrict__ perm, int32_t *__restrict__ pos, int32_t *__restrict__ blocks,
                    int block_rows) {
    __shared__ moe::PermShared sh;
    moe::permute_block(sh, rid, n_pairs, g_self, C, slot_count, slot_off, perm, pos, blocks, block_rows);
}

// The dispatch of a shared expert: one slot that every token visits once (identity permutation),
// cut into the same blocks of rows as any other slot.
__global__ __launch_bounds__(256)
void shared_dispatch_kernel(int T, int block_rows, int32_t *__restrict__ slot_off, int32_t *__restrict__ perm,
                            int32_t *__restrict__ blocks) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x, n = gridDim.x * blockDim.x;
    const int n_blocks = (T + block_rows - 1) / block_rows;
    if (tid == 0) {
        slot_off[0] = 0;
        slot_off[1] = T;
        reinterpret_cast<int4 *>(blocks)[0] = make_int4(n_blocks, block_rows, T > 64 ? (T + 63) / 64 : 0, T > 64 ? (T + 127) / 128 : 0);
    }
    for (int i = tid; i < T; i += n) perm[i] = i;
    for (int b = tid; b < n_blocks; b += n) reinterpret_cast<int4 *>(blocks)[1 + b] = make_int4(0, b * block_rows, T, 0);
}

// One workgroup per (token, 1024-column chunk); each thread owns 4 consecutive columns.
// Ys (optional): rows of a shared expert's output, added with weight 1 after the routed sum.
template <bool OUT_BF16>
__global__ __launch_bounds__(256)
void combine_kernel(const float *__restrict__ Yp, const int32_t *__restrict__ pos,
                    const float *__restrict__ w, const float *__restrict__ Ys, int k, int d_h, void *__restrict__ Y) {
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
    if (Ys) {
        const float4 y = *reinterpret_cast<const float4 *>(Ys + static_cast<size_t>(i) * d_h + col);
        acc.x += y.x; acc.y += y.y; acc.z += y.z; acc.w += y.w;
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
                           int32_t *pos_dev, int32_t *blocks_dev, void *stream) {
    if (!pl || T < 0 || k < 1) return MOE_EINVAL;
    if (g_self < 0 || g_self >= pl->n_inst) return MOE_EINVAL;
    if (k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (static_cast<long long>(T) * k > 0x7fffffffLL) return MOE_ESHAPE;
    if (!slot_count_dev || !slot_off_dev || !blocks_dev) return MOE_EINVAL;
    if (T > 0 && (!rid_dev || !perm_dev || !pos_dev)) return MOE_EINVAL;
    if (!moe::aligned(rid_dev, 4) || !moe::aligned(slot_count_dev, 4) || !moe::aligned(slot_off_dev, 4) ||
        !moe::aligned(perm_dev, 4) || !moe::aligned(pos_dev, 4) || !moe::aligned(blocks_dev, 16))
        return MOE_EINVAL;
    hipLaunchKernelGGL(permute_kernel, dim3(1), dim3(kPermThreads), 0, static_cast<hipStream_t>(stream),
                       rid_dev, T * k, g_self, pl->C, slot_count_dev, slot_off_dev, perm_dev, pos_dev, blocks_dev,
                       moe::ffn_block_rows(T));
    return moe::check_launch("moe_permute");
}

extern "C" size_t moe_max_blocks(int T, int k, int C) {
    if (T < 0 || k < 1 || C < 1) return 0;
    return static_cast<size_t>(moe::ffn_max_blocks(T, k, C));
}

extern "C" int moe_block_rows(int T) { return T < 0 ? 0 : moe::ffn_block_rows(T); }

extern "C" size_t moe_block_list_len(int T, int k, int C) {
    if (T < 0 || k < 1 || C < 1) return 0;
    return 4 * (1 + static_cast<size_t>(moe::ffn_max_blocks(T, k, C)));
}

namespace {

int combine(const float *Yp_dev, const int32_t *pos_dev, const float *topk_w_dev, const float *Ys_dev, bool shared,
            int T, int k, int d_h, int dtype, void *Y_dev, void *stream, const char *what) {
    if (T < 0 || k < 1 || d_h < 1) return MOE_EINVAL;
    if (dtype != MOE_DTYPE_BF16 && dtype != MOE_DTYPE_F32) return MOE_EINVAL;
    if (d_h % 4 != 0 || k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (T == 0) return MOE_OK;
    if (!Yp_dev || !pos_dev || !topk_w_dev || !Y_dev || (shared && !Ys_dev)) return MOE_EINVAL;
    if (!moe::aligned(Yp_dev, 16) || !moe::aligned(pos_dev, 4) || !moe::aligned(topk_w_dev, 4) ||
        !moe::aligned(Ys_dev, 16) || !moe::aligned(Y_dev, dtype == MOE_DTYPE_BF16 ? 8 : 16))
        return MOE_EINVAL;
    const dim3 grid(T, (d_h + 1023) / 1024);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == MOE_DTYPE_BF16)
        hipLaunchKernelGGL(combine_kernel<true>, grid, dim3(256), 0, st, Yp_dev, pos_dev, topk_w_dev, Ys_dev, k, d_h, Y_dev);
    else
        hipLaunchKernelGGL(combine_kernel<false>, grid, dim3(256), 0, st, Yp_dev, pos_dev, topk_w_dev, Ys_dev, k, d_h, Y_dev);
    return moe::check_launch(what);
}

}  // namespace

extern "C" int moe_combine(const float *Yp_dev, const int32_t *pos_dev, const float *topk_w_dev,
                           int T, int k, int d_h, int dtype, void *Y_dev, void *stream) {
    return combine(Yp_dev, pos_dev, topk_w_dev, nullptr, false, T, k, d_h, dtype, Y_dev, stream, "moe_combine");
}

extern "C" int moe_combine_shared(const float *Yp_dev, const int32_t *pos_dev, const float *topk_w_dev,
                                  const float *Ys_dev, int T, int k, int d_h, int dtype, void *Y_dev, void *stream) {
    return combine(Yp_dev, pos_dev, topk_w_dev, Ys_dev, true, T, k, d_h, dtype, Y_dev, stream, "moe_combine_shared");
}

extern "C" int moe_shared_dispatch(int T, int32_t *slot_off_dev, int32_t *perm_dev, int32_t *blocks_dev, void *stream) {
    if (T < 0 || !slot_off_dev || !blocks_dev || (T > 0 && !perm_dev)) return MOE_EINVAL;
    if (!moe::aligned(slot_off_dev, 4) || !moe::aligned(perm_dev, 4) || !moe::aligned(blocks_dev, 16)) return MOE_EINVAL;
    const int grid = T > 256 ? (T + 255) / 256 < 64 ? (T + 255) / 256 : 64 : 1;
    hipLaunchKernelGGL(shared_dispatch_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream), T,
                       moe::ffn_block_rows(T), slot_off_dev, perm_dev, blocks_dev);
    return moe::check_launch("moe_shared_dispatch");
}
