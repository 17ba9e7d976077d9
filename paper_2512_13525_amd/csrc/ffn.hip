// a5: grouped expert FFN over the activated experts only (Janus Sec. 2.2: an expert is a
// fused gate/up GEMM and a down GEMM; at decode sizes the layer is bound by streaming the
// activated experts' weights from HBM, so latency follows the activated-expert count).
//
// bf16 path.  Weights are consumed in a tile-packed layout: every 16-row x 32-column tile
// of a weight matrix is stored as the 1 KiB image of the MFMA A-operand of one wavefront
// (lane l holds row l%16, columns (l/16)*8 .. +7), so a wavefront streams its tiles with
// fully coalesced 128-bit loads straight into MFMA registers.  Tokens are the B operand
// (lane l holds token l%16, the same 8 columns), gathered through `perm`; the 16x16 fp32
// result tile leaves lane l with 4 consecutive output channels (l/16)*4.. of token l%16.
//
//   stage 1  gateup_kernel: workgroup = (slot, 16 intermediate channels); its 4 wavefronts
//            split K = d_h, partial tiles meet in LDS, SiLU(gate)*up is rounded to bf16 once
//            and written to the workspace `act` [n_local, d_e].
//   stage 2  down_kernel: wavefront = (slot, 16 output channels) over K = d_e, reading `act`.
// Workgroups of slots without requests leave at once; their weights are never touched.
//
// fp32 path (correctness configuration): plain wave-per-output-row dot products.
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kTokTiles = 4;          // token tiles (of 16) a workgroup keeps in registers per pass

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// ------------------------------------------------------------------ packing
// W13 [C, 2*d_e, d_h] -> [C][d_e/16][d_h/32][2 (gate, up)][64 lanes][8]
__global__ void pack_w13_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                int C, int d_h, int d_e) {
    const int JT = d_e / 16, KS = d_h / 32;
    const size_t n = static_cast<size_t>(C) * JT * KS * 2 * 64;
    for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < n;
         i += static_cast<size_t>(gridDim.x) * blockDim.x) {
        const int lane = i % 64;
        size_t r = i / 64;
        const int gu = r % 2; r /= 2;
        const int kk = r % KS; r /= KS;
        const int jt = r % JT;
        const int s = r / JT;
        const size_t row = static_cast<size_t>(s) * 2 * d_e + static_cast<size_t>(gu) * d_e + jt * 16 + (lane & 15);
        const size_t col = static_cast<size_t>(kk) * 32 + (lane >> 4) * 8;
        dst[i] = src[(row * d_h + col) / 8];
    }
}

// W2 [C, d_h, d_e] -> [C][d_h/16][d_e/32][64 lanes][8]
__global__ void pack_w2_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                               int C, int d_h, int d_e) {
    const int IT = d_h / 16, KS = d_e / 32;
    const size_t n = static_cast<size_t>(C) * IT * KS * 64;
    for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < n;
         i += static_cast<size_t>(gridDim.x) * blockDim.x) {
        const int lane = i % 64;
        size_t r = i / 64;
        const int kk = r % KS; r /= KS;
        const int it = r % IT;
        const int s = r / IT;
        const size_t row = static_cast<size_t>(s) * d_h + it * 16 + (lane & 15);
        const size_t col = static_cast<size_t>(kk) * 32 + (lane >> 4) * 8;
        dst[i] = src[(row * d_e + col) / 8];
    }
}

// ------------------------------------------------------------------ stage 1 (bf16)
template <int NT>
__device__ __forceinline__ void gateup_accumulate(const bf16x8 *__restrict__ wp, const uint16_t *const *xp,
                                                  int k_begin, int k_end, f32x4 *acc_g, f32x4 *acc_u) {
#pragma unroll 4
    for (int kk = k_begin; kk < k_end; ++kk) {
        const bf16x8 a_g = wp[(static_cast<size_t>(kk) * 2 + 0) * 64];
        const bf16x8 a_u = wp[(static_cast<size_t>(kk) * 2 + 1) * 64];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const bf16x8 b = *reinterpret_cast<const bf16x8 *>(xp[t] + kk * 32);
            acc_g[t] = mfma16(a_g, b, acc_g[t]);
            acc_u[t] = mfma16(a_u, b, acc_u[t]);
        }
    }
}

__global__ __launch_bounds__(256)
void gateup_kernel(const uint16_t *__restrict__ X, const bf16x8 *__restrict__ W13p,
                   const int32_t *__restrict__ slot_off, const int32_t *__restrict__ perm,
                   uint16_t *__restrict__ act, int k, int d_h, int d_e) {
    __shared__ f32x4 red[4][kTokTiles][2][64];          // [wave][token tile][gate|up][lane]
    const int jt = blockIdx.x, s = blockIdx.y;
    const int lo = slot_off[s];
    const int m = slot_off[s + 1] - lo;
    if (m <= 0) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = lane & 15, q = lane >> 4;
    const int JT = d_e / 16, KS = d_h / 32;
    const int k_begin = wave * KS / 4, k_end = (wave + 1) * KS / 4;
    const bf16x8 *wp = W13p + (static_cast<size_t>(s) * JT + jt) * KS * 2 * 64 + lane;
    const int n_tiles = (m + 15) / 16;

    for (int tile0 = 0; tile0 < n_tiles; tile0 += kTokTiles) {
        const int nt = min(kTokTiles, n_tiles - tile0);
        const uint16_t *xp[kTokTiles];
#pragma unroll
        for (int t = 0; t < kTokTiles; ++t) {
            const int idx = (tile0 + t) * 16 + n;
            const int tok = perm[lo + (idx < m ? idx : 0)] / k;     // padding lanes reuse a valid row
            xp[t] = X + static_cast<size_t>(tok) * d_h + q * 8;
        }
        f32x4 acc_g[kTokTiles], acc_u[kTokTiles];
#pragma unroll
        for (int t = 0; t < kTokTiles; ++t) { acc_g[t] = f32x4{0, 0, 0, 0}; acc_u[t] = f32x4{0, 0, 0, 0}; }
        switch (nt) {
            case 1: gateup_accumulate<1>(wp, xp, k_begin, k_end, acc_g, acc_u); break;
            case 2: gateup_accumulate<2>(wp, xp, k_begin, k_end, acc_g, acc_u); break;
            case 3: gateup_accumulate<3>(wp, xp, k_begin, k_end, acc_g, acc_u); break;
            default: gateup_accumulate<4>(wp, xp, k_begin, k_end, acc_g, acc_u); break;
        }
#pragma unroll
        for (int t = 0; t < kTokTiles; ++t) {
            if (t < nt) { red[wave][t][0][lane] = acc_g[t]; red[wave][t][1][lane] = acc_u[t]; }
        }
        __syncthreads();
        if (wave < nt) {                                 // wave t finishes token tile t
            const int t = wave;
            f32x4 g = red[0][t][0][lane], u = red[0][t][1][lane];
#pragma unroll
            for (int w = 1; w < 4; ++w) { g += red[w][t][0][lane]; u += red[w][t][1][lane]; }
            const int idx = (tile0 + t) * 16 + n;
            if (idx < m) {
                ushort4 o;
                o.x = moe::f32_to_bf16(g[0] / (1.0f + __expf(-g[0])) * u[0]);
                o.y = moe::f32_to_bf16(g[1] / (1.0f + __expf(-g[1])) * u[1]);
                o.z = moe::f32_to_bf16(g[2] / (1.0f + __expf(-g[2])) * u[2]);
                o.w = moe::f32_to_bf16(g[3] / (1.0f + __expf(-g[3])) * u[3]);
                *reinterpret_cast<ushort4 *>(act + static_cast<size_t>(lo + idx) * d_e + jt * 16 + q * 4) = o;
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------ stage 2 (bf16)
template <int NT>
__device__ __forceinline__ void down_accumulate(const bf16x8 *__restrict__ wp, const uint16_t *const *ap,
                                                int KS, f32x4 *acc) {
#pragma unroll 4
    for (int kk = 0; kk < KS; ++kk) {
        const bf16x8 a = wp[static_cast<size_t>(kk) * 64];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const bf16x8 b = *reinterpret_cast<const bf16x8 *>(ap[t] + kk * 32);
            acc[t] = mfma16(a, b, acc[t]);
        }
    }
}

__global__ __launch_bounds__(256)
void down_kernel(const uint16_t *__restrict__ act, const bf16x8 *__restrict__ W2p,
                 const int32_t *__restrict__ slot_off, float *__restrict__ Yp, int d_h, int d_e) {
    const int s = blockIdx.y;
    const int lo = slot_off[s];
    const int m = slot_off[s + 1] - lo;
    if (m <= 0) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = lane & 15, q = lane >> 4;
    const int IT = d_h / 16, KS = d_e / 32;
    const int it = blockIdx.x * 4 + wave;
    if (it >= IT) return;                                // no block barrier below
    const bf16x8 *wp = W2p + (static_cast<size_t>(s) * IT + it) * KS * 64 + lane;
    const int n_tiles = (m + 15) / 16;

    for (int tile0 = 0; tile0 < n_tiles; tile0 += kTokTiles) {
        const int nt = min(kTokTiles, n_tiles - tile0);
        const uint16_t *ap[kTokTiles];
#pragma unroll
        for (int t = 0; t < kTokTiles; ++t) {
            const int idx = (tile0 + t) * 16 + n;
            ap[t] = act + static_cast<size_t>(lo + (idx < m ? idx : 0)) * d_e + q * 8;
        }
        f32x4 acc[kTokTiles];
#pragma unroll
        for (int t = 0; t < kTokTiles; ++t) acc[t] = f32x4{0, 0, 0, 0};
        switch (nt) {
            case 1: down_accumulate<1>(wp, ap, KS, acc); break;
            case 2: down_accumulate<2>(wp, ap, KS, acc); break;
            case 3: down_accumulate<3>(wp, ap, KS, acc); break;
            default: down_accumulate<4>(wp, ap, KS, acc); break;
        }
#pragma unroll
        for (int t = 0; t < kTokTiles; ++t) {
            const int idx = (tile0 + t) * 16 + n;
            if (t < nt && idx < m)
                *reinterpret_cast<f32x4 *>(Yp + static_cast<size_t>(lo + idx) * d_h + it * 16 + q * 4) = acc[t];
        }
    }
}

// ------------------------------------------------------------------ fp32 path
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, MOE_WAVE);
    return v;
}

// grid (ceil(d_e/4), T*k rows): wave w of a block computes act[r, c] for c = blockIdx.x*4 + w
__global__ __launch_bounds__(256)
void gateup_f32_kernel(const float *__restrict__ X, const float *__restrict__ W13,
                       const int32_t *__restrict__ slot_off, const int32_t *__restrict__ perm,
                       float *__restrict__ act, int C, int k, int d_h, int d_e) {
    const int r = blockIdx.y;
    if (r >= slot_off[C]) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + wave;
    if (c >= d_e) return;
    int s = 0;
    while (slot_off[s + 1] <= r) ++s;                    // slot of row r (C is small)
    const int tok = perm[r] / k;
    const float *x = X + static_cast<size_t>(tok) * d_h;
    const float *wg = W13 + (static_cast<size_t>(s) * 2 * d_e + c) * d_h;
    const float *wu = wg + static_cast<size_t>(d_e) * d_h;
    float h = 0.f, u = 0.f;
    for (int i = lane * 4; i < d_h; i += 256) {
        const float4 xv = *reinterpret_cast<const float4 *>(x + i);
        const float4 gv = *reinterpret_cast<const float4 *>(wg + i);
        const float4 uv = *reinterpret_cast<const float4 *>(wu + i);
        h += xv.x * gv.x + xv.y * gv.y + xv.z * gv.z + xv.w * gv.w;
        u += xv.x * uv.x + xv.y * uv.y + xv.z * uv.z + xv.w * uv.w;
    }
    h = wave_sum(h);
    u = wave_sum(u);
    if (lane == 0) act[static_cast<size_t>(r) * d_e + c] = h / (1.0f + expf(-h)) * u;
}

__global__ __launch_bounds__(256)
void down_f32_kernel(const float *__restrict__ act, const float *__restrict__ W2,
                     const int32_t *__restrict__ slot_off, float *__restrict__ Yp, int C, int d_h, int d_e) {
    const int r = blockIdx.y;
    if (r >= slot_off[C]) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + wave;
    if (c >= d_h) return;
    int s = 0;
    while (slot_off[s + 1] <= r) ++s;
    const float *a = act + static_cast<size_t>(r) * d_e;
    const float *wd = W2 + (static_cast<size_t>(s) * d_h + c) * d_e;
    float y = 0.f;
    for (int i = lane * 4; i < d_e; i += 256) {
        const float4 av = *reinterpret_cast<const float4 *>(a + i);
        const float4 wv = *reinterpret_cast<const float4 *>(wd + i);
        y += av.x * wv.x + av.y * wv.y + av.z * wv.z + av.w * wv.w;
    }
    y = wave_sum(y);
    if (lane == 0) Yp[static_cast<size_t>(r) * d_h + c] = y;
}

}  // namespace

extern "C" size_t moe_workspace_bytes(int T, int k, int C, int d_h, int d_e, int dtype) {
    (void)C; (void)d_h;
    if (T < 0 || k < 1 || d_e < 1) return 0;
    const size_t elt = dtype == MOE_DTYPE_F32 ? 4 : 2;
    const size_t bytes = static_cast<size_t>(T) * k * d_e * elt;
    return (bytes + 255) / 256 * 256 + 256;
}

extern "C" int moe_pack_weights_bf16(const void *W13_dev, const void *W2_dev, int C, int d_h, int d_e,
                                     void *W13_packed_dev, void *W2_packed_dev, void *stream) {
    if (C < 1 || d_h < 1 || d_e < 1) return MOE_EINVAL;
    if (C > MOE_MAX_SLOTS || d_h % 32 != 0 || d_e % 32 != 0) return MOE_ESHAPE;
    if (!W13_dev || !W2_dev || !W13_packed_dev || !W2_packed_dev) return MOE_EINVAL;
    if (!moe::aligned(W13_dev, 16) || !moe::aligned(W2_dev, 16) || !moe::aligned(W13_packed_dev, 16) ||
        !moe::aligned(W2_packed_dev, 16))
        return MOE_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(pack_w13_kernel, dim3(2048), dim3(256), 0, st,
                       static_cast<const uint4 *>(W13_dev), static_cast<uint4 *>(W13_packed_dev), C, d_h, d_e);
    hipLaunchKernelGGL(pack_w2_kernel, dim3(2048), dim3(256), 0, st,
                       static_cast<const uint4 *>(W2_dev), static_cast<uint4 *>(W2_packed_dev), C, d_h, d_e);
    return moe::check_launch("moe_pack_weights_bf16");
}

extern "C" int moe_grouped_ffn(const void *X_dev, const void *W13_dev, const void *W2_dev,
                               int T, int k, int C, int d_h, int d_e, int dtype,
                               const int32_t *slot_off_dev, const int32_t *perm_dev,
                               float *Yp_dev, void *workspace_dev, size_t workspace_bytes, void *stream) {
    if (T < 0 || k < 1 || C < 1 || d_h < 1 || d_e < 1) return MOE_EINVAL;
    if (dtype != MOE_DTYPE_BF16 && dtype != MOE_DTYPE_F32) return MOE_EINVAL;
    if (C > MOE_MAX_SLOTS || k > MOE_MAX_TOPK) return MOE_ESHAPE;
    if (static_cast<long long>(T) * k > 0x7fffffffLL) return MOE_ESHAPE;
    if (dtype == MOE_DTYPE_BF16 && (d_h % 32 != 0 || d_e % 32 != 0)) return MOE_ESHAPE;
    if (dtype == MOE_DTYPE_F32 && (d_h % 4 != 0 || d_e % 4 != 0)) return MOE_ESHAPE;
    if (T == 0) return MOE_OK;
    if (!X_dev || !W13_dev || !W2_dev || !slot_off_dev || !perm_dev || !Yp_dev || !workspace_dev) return MOE_EINVAL;
    if (!moe::aligned(X_dev, 16) || !moe::aligned(W13_dev, 16) || !moe::aligned(W2_dev, 16) ||
        !moe::aligned(Yp_dev, 16) || !moe::aligned(workspace_dev, 256) || !moe::aligned(slot_off_dev, 4) ||
        !moe::aligned(perm_dev, 4))
        return MOE_EINVAL;
    if (workspace_bytes < moe_workspace_bytes(T, k, C, d_h, d_e, dtype)) return MOE_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == MOE_DTYPE_BF16) {
        uint16_t *act = static_cast<uint16_t *>(workspace_dev);
        hipLaunchKernelGGL(gateup_kernel, dim3(d_e / 16, C), dim3(256), 0, st,
                           static_cast<const uint16_t *>(X_dev), static_cast<const bf16x8 *>(W13_dev),
                           slot_off_dev, perm_dev, act, k, d_h, d_e);
        hipLaunchKernelGGL(down_kernel, dim3((d_h / 16 + 3) / 4, C), dim3(256), 0, st,
                           act, static_cast<const bf16x8 *>(W2_dev), slot_off_dev, Yp_dev, d_h, d_e);
    } else {
        // one grid row per possible request row; rows >= n_local leave at once
        const long long rows = static_cast<long long>(T) * k;
        if (rows > 65535) return MOE_ESHAPE;
        float *act = static_cast<float *>(workspace_dev);
        hipLaunchKernelGGL(gateup_f32_kernel, dim3((d_e + 3) / 4, rows), dim3(256), 0, st,
                           static_cast<const float *>(X_dev), static_cast<const float *>(W13_dev),
                           slot_off_dev, perm_dev, act, C, k, d_h, d_e);
        hipLaunchKernelGGL(down_f32_kernel, dim3((d_h + 3) / 4, rows), dim3(256), 0, st,
                           act, static_cast<const float *>(W2_dev), slot_off_dev, Yp_dev, C, d_h, d_e);
    }
    return moe::check_launch("moe_grouped_ffn");
}
