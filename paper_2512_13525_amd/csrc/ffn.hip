// a5: grouped expert FFN over the activated experts only (Janus Sec. 2.2: an expert is a
// fused gate/up GEMM and a down GEMM; at decode sizes the layer is bound by streaming the
// activated experts' weights from HBM, so latency follows the activated-expert count).
//
// This file: the weight packing, the workspace, the fp32 correctness path and the C entry
// point.  The bf16 kernels are in ffn_stream.hip.
//
// bf16 weights are consumed in a tile-packed layout: a 16-row x 32-column tile of a weight
// matrix is stored as the 1 KiB image of the MFMA A-operand of one wavefront (lane l holds row
// l%16, columns (l/16)*8 .. +7), and the two 16-row tiles a workgroup multiplies together (16
// gate + 16 up channels in stage 1, 32 output channels in stage 2) alternate per K-step, so a
// workgroup's share of a matrix is one contiguous run of 2 KiB steps read with fully coalesced
// 128-bit loads straight into MFMA registers.
//
// fp32 path (correctness configuration): plain wave-per-output-row dot products, two kernels.
#include <stdlib.h>

#include <mutex>

#include "common.h"

namespace {

// Workspace layout (bytes):
//   [0, kCtrlBytes)      control words, zeroed by moe_workspace_init and left zero by every call:
//                        int [1] = error word, then the per-block hand-off counters of the bf16
//                        kernels (see ffn_stream.hip)
//   [kCtrlBytes, ...)    act: SiLU(gate)*up of every local request row (fp32: [row][d_e];
//                        bf16: one region per entry of the work list, see ffn_stream.hip)
constexpr size_t kCtrlBytes = moe::kFfnCtrlBytes;

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

// W2 [C, d_h, d_e] -> [C][d_h/32][d_e/32][2 (rows 0-15, rows 16-31)][64 lanes][8]
__global__ void pack_w2_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                               int C, int d_h, int d_e) {
    const int IT = d_h / 32, KS = d_e / 32;
    const size_t n = static_cast<size_t>(C) * IT * KS * 2 * 64;
    for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < n;
         i += static_cast<size_t>(gridDim.x) * blockDim.x) {
        const int lane = i % 64;
        size_t r = i / 64;
        const int half = r % 2; r /= 2;
        const int kk = r % KS; r /= KS;
        const int it = r % IT;
        const int s = r / IT;
        const size_t row = static_cast<size_t>(s) * d_h + it * 32 + half * 16 + (lane & 15);
        const size_t col = static_cast<size_t>(kk) * 32 + (lane >> 4) * 8;
        dst[i] = src[(row * d_e + col) / 8];
    }
}

__global__ void fill_zero_kernel(int *p, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0;
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

namespace {
__global__ void set_word_kernel(int *p, int v) { *p = v; }
}  // namespace

extern "C" int moe_workspace_set_option(void *workspace_dev, size_t workspace_bytes, int option, int value, void *stream) {
    if (!workspace_dev || !moe::aligned(workspace_dev, 256)) return MOE_EINVAL;
    if (workspace_bytes < kCtrlBytes) return MOE_EWORKSPACE;
    if (value < 0) return MOE_EINVAL;
    int word;
    if (option == MOE_WS_OPT_SPIN_LIMIT) word = moe::kCtrlSpinLimit;
    else if (option == MOE_WS_OPT_WIDE_MIN_WORKGROUPS) word = moe::kCtrlWideMin;
    else return MOE_EINVAL;
    hipLaunchKernelGGL(set_word_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream),
                       static_cast<int *>(workspace_dev) + word, value);
    return moe::check_launch("moe_workspace_set_option");
}

extern "C" size_t moe_workspace_bytes(int T, int k, int C, int d_h, int d_e, int dtype) {
    (void)d_h;
    if (T < 0 || k < 1 || C < 1 || d_e < 1) return 0;
    // fp32: one row per request; bf16: whole blocks of rows (at most C partly filled ones)
    const size_t bytes = dtype == MOE_DTYPE_F32
        ? static_cast<size_t>(T) * k * d_e * 4
        : moe::ffn_stream_act_bytes(T, k, C, d_e) + (moe::ffn_has_gemm(T) ? static_cast<size_t>(T) * k * d_e * 2 : 0);
    return kCtrlBytes + (bytes + 255) / 256 * 256 + 256;
}

extern "C" int moe_workspace_init(void *workspace_dev, size_t workspace_bytes, void *stream) {
    if (!workspace_dev || !moe::aligned(workspace_dev, 256)) return MOE_EINVAL;
    if (workspace_bytes < kCtrlBytes) return MOE_EWORKSPACE;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(64), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<int *>(workspace_dev), static_cast<int>(kCtrlBytes / 4));
    return moe::check_launch("moe_workspace_init");
}

extern "C" int moe_workspace_status(const void *workspace_dev, int *status_host) {
    if (!workspace_dev || !status_host) return MOE_EINVAL;
    int hdr[2] = {0, 0};
    hipError_t e = hipMemcpy(hdr, workspace_dev, sizeof(hdr), hipMemcpyDeviceToHost);
    if (e != hipSuccess) { moe::set_hip_error(e, "moe_workspace_status"); return MOE_EHIP; }
    *status_host = hdr[moe::kCtrlStatus];
    return MOE_OK;
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

namespace {

int grouped_ffn(const void *X_dev, const void *W13_dev, const void *W2_dev,
                int T, int k, int C, int d_h, int d_e, int dtype,
                const int32_t *slot_off_dev, const int32_t *perm_dev, const int32_t *blocks_dev,
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
    if (dtype == MOE_DTYPE_BF16 && (!blocks_dev || !moe::aligned(blocks_dev, 16))) return MOE_EINVAL;
    if (workspace_bytes < moe_workspace_bytes(T, k, C, d_h, d_e, dtype)) return MOE_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace_dev);
    if (dtype == MOE_DTYPE_BF16) {
        // the kernels address token rows with 32-bit byte offsets
        if (static_cast<long long>(T) * d_h * 2 > 0xffffffffLL) return MOE_ESHAPE;
        if (moe::ffn_has_gemm(T)) {
            uint16_t *act_rows = reinterpret_cast<uint16_t *>(ws + kCtrlBytes + moe::ffn_stream_act_bytes(T, k, C, d_e));
            const int rcw = moe::launch_ffn_wide(X_dev, W13_dev, W2_dev, T, k, C, d_h, d_e, blocks_dev,
                                                 perm_dev, reinterpret_cast<const int *>(ws), act_rows, Yp_dev, st);
            if (rcw != MOE_OK) return rcw;
        }
        const int rc = moe::launch_ffn_stream(X_dev, W13_dev, W2_dev, T, k, C, d_h, d_e, blocks_dev, perm_dev,
                                              reinterpret_cast<int *>(ws), reinterpret_cast<uint16_t *>(ws + kCtrlBytes),
                                              Yp_dev, st);
        if (rc != MOE_OK) return rc;
    } else {
        // one grid row per possible request row; rows >= n_local leave at once
        const long long rows = static_cast<long long>(T) * k;
        if (rows > 65535) return MOE_ESHAPE;
        float *act = reinterpret_cast<float *>(ws + kCtrlBytes);
        hipLaunchKernelGGL(gateup_f32_kernel, dim3((d_e + 3) / 4, rows), dim3(256), 0, st,
                           static_cast<const float *>(X_dev), static_cast<const float *>(W13_dev),
                           slot_off_dev, perm_dev, act, C, k, d_h, d_e);
        hipLaunchKernelGGL(down_f32_kernel, dim3((d_h + 3) / 4, rows), dim3(256), 0, st,
                           act, static_cast<const float *>(W2_dev), slot_off_dev, Yp_dev, C, d_h, d_e);
    }
    return moe::check_launch("moe_grouped_ffn");
}

// Scratch of moe_grouped_ffn_static: one copy per GPU, held until the process ends.  In host code
// this name is only a handle for hipGetSymbolAddress; the kernels get the address it returns.
constexpr size_t kStaticScratchBytes = MOE_FFN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];        // device address of `scratch` on each GPU, looked up once per GPU

// Address of this GPU's copy of the scratch array (the current device's), or null with the HIP error recorded.
void *static_scratch() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        moe::set_hip_error(e != hipSuccess ? e : hipErrorInvalidDevice, "moe_grouped_ffn_static: hipGetDevice");
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            moe::set_hip_error(e != hipSuccess ? e : hipErrorInvalidSymbol, "moe_grouped_ffn_static: hipGetSymbolAddress");
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" int moe_grouped_ffn(const void *X_dev, const void *W13_dev, const void *W2_dev,
                               int T, int k, int C, int d_h, int d_e, int dtype,
                               const int32_t *slot_off_dev, const int32_t *perm_dev, const int32_t *blocks_dev,
                               float *Yp_dev, void *workspace_dev, size_t workspace_bytes, void *stream) {
    return grouped_ffn(X_dev, W13_dev, W2_dev, T, k, C, d_h, d_e, dtype, slot_off_dev, perm_dev, blocks_dev, Yp_dev,
                       workspace_dev, workspace_bytes, stream);
}

extern "C" int moe_grouped_ffn_static(const void *X_dev, const void *W13_dev, const void *W2_dev,
                                      int T, int k, int C, int d_h, int d_e, int dtype,
                                      const int32_t *slot_off_dev, const int32_t *perm_dev, const int32_t *blocks_dev,
                                      float *Yp_dev, void *stream) {
    if (T < 0 || k < 1 || C < 1 || d_h < 1 || d_e < 1) return MOE_EINVAL;
    if (dtype != MOE_DTYPE_BF16 && dtype != MOE_DTYPE_F32) return MOE_EINVAL;
    if (static_cast<long long>(T) * k > 0x7fffffffLL) return MOE_ESHAPE;
    // the size the allocating entry point would ask its caller for must fit the fixed array
    const size_t need = moe_workspace_bytes(T, k, C, d_h, d_e, dtype);
    if (need == 0 || need > kStaticScratchBytes) return MOE_EWORKSPACE;
    if (T == 0) return MOE_OK;
    void *ws = static_scratch();
    if (!ws) return MOE_EHIP;
    // The array keeps what the last call on this GPU left: the header (status word, options) and the
    // hand-off lines of every block this call can have must start at zero.  A fill kernel, not a
    // memset node, so that the call can be captured into a graph.
    if (dtype == MOE_DTYPE_BF16) {
        const long long lines = 1 + moe::ffn_max_blocks(T, k, C);
        if (lines * 1024 > static_cast<long long>(kCtrlBytes)) return MOE_ESHAPE;
        hipLaunchKernelGGL(fill_zero_kernel, dim3(static_cast<unsigned>((lines + 3) / 4)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), static_cast<int *>(ws), static_cast<int>(lines * 256));
    }
    return grouped_ffn(X_dev, W13_dev, W2_dev, T, k, C, d_h, d_e, dtype, slot_off_dev, perm_dev, blocks_dev, Yp_dev,
                       ws, kStaticScratchBytes, stream);
}
