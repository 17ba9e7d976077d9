// Internal helpers shared by the translation units of libmoe_janus (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "moe_janus.h"

#define MOE_WAVE 64

struct moe_placement {
    int E, n_inst, C;
    int n_words;                 // ceil(E/64): 64-bit words of an expert bitset
    // host tables
    int32_t *slot_to_expert_h;   // [n_inst*C]
    int32_t *R_h;                // [E]
    // device tables (one allocation, 256-byte aligned sub-arrays)
    void     *dev_block;
    uint64_t *host_mask_d;       // [E]  bit g set <=> instance g hosts a replica of e
    int16_t  *slot_of_d;         // [E*n_inst] local slot of e on g, -1 if not hosted
    int32_t  *single_rid_d;      // [E]  RID when R(e) == 1, else -1
    uint64_t *multi_mask_d;      // [n_words] bit e set <=> R(e) > 1
    uint64_t *single_mask_d;     // [n_inst*n_words] single-replica experts hosted on g
    int device;
};

namespace moe {

void set_hip_error(hipError_t e, const char *where);

inline int check_launch(const char *where) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_hip_error(e, where);
        return MOE_EHIP;
    }
    return MOE_OK;
}

// Control region at the start of the FFN workspace: a header of 256 ints, then the hand-off counters
// of the blocks (ffn_stream.hip).  Header words: the status bits, and the per-workspace options
// that moe_workspace_set_option writes and moe_workspace_init resets to 0 (= the default).
constexpr size_t kFfnCtrlBytes = 4u << 20;
constexpr int kCtrlStatus = 1;           // bit 0: a wait overran; bit 1: list cut for another block size
constexpr int kCtrlSpinLimit = 2;        // polls a stage-2 workgroup spends on a block's flag before it gives up
constexpr int kCtrlWideMin = 3;          // workgroups of wide blocks a batch must have for them to be used (ffn_stream.hip)

// Blocks of the work list that get workgroups of their own in the streaming launch (longer lists wrap around)
constexpr unsigned kFfnLaneBlocks = 128;

// Request rows per block of the FFN work list: small batches take blocks of 32 rows (more, shorter
// workgroups), larger ones blocks of 64 (hot slots then re-read their expert half as often).
inline int ffn_block_rows(int T) { return T < 384 ? 32 : MOE_FFN_BLOCK_ROWS; }

// Upper bound of the number of blocks over all slots, whatever the requests are (also when a
// token names one expert several times): every slot has at most one partly filled block, and
// the full ones hold T*k requests at most.
inline long long ffn_max_blocks(int T, int k, int C) {
    return C + static_cast<long long>(T) * k / ffn_block_rows(T);
}

// Bytes of the intermediate `act` per entry of the work list: a block of rows x d_e rounded up to
// whole 128-byte lines (64 channels).  A wide block (ffn_stream.hip) uses the regions of the entries
// it spans.
inline size_t ffn_act_block_bytes(int T, int d_e) {
    return static_cast<size_t>(ffn_block_rows(T)) * ((d_e + 63) / 64 * 64) * 2;
}
inline size_t ffn_stream_act_bytes(int T, int k, int C, int d_e) {
    const size_t b = static_cast<size_t>(ffn_max_blocks(T, k, C)) * ffn_act_block_bytes(T, d_e);
    return (b + 255) / 256 * 256;
}

// bf16 grouped FFN (ffn_stream.hip); shapes validated by the caller.  `ctrl` is the zero-initialised
// control region of the workspace, `act` holds ffn_stream_act_bytes(T, k, C, d_e) bytes.  Returns MOE_OK
// or MOE_ESHAPE (too many blocks).
int launch_ffn_stream(const void *X, const void *W13p, const void *W2p, int T, int k, int C, int d_h, int d_e,
                      const int32_t *blocks, const int32_t *perm, int *ctrl, uint16_t *act,
                      float *Yp, hipStream_t st);

// Batches of at least kGemmMinTokens tokens: slots with more than 64 requests as blocks of 128 rows in
// two tiled-GEMM launches of their own (ffn_wide.hip, three workgroups of 168 registers per CU),
// when the list counts enough 128-row blocks (header word 3) for kGemmMinWorkgroups first-stage
// workgroups; the streaming launch then skips those slots.  Every kernel takes the decision from
// the list's header in the same way.  `act_rows` holds T*k rows of d_e bf16 behind the streaming
// launch's intermediate.
constexpr int kGemmMinTokens = 2048;
inline bool ffn_has_gemm(int T) { return T >= kGemmMinTokens; }
constexpr int kGemmMinWorkgroups = 512;
constexpr int kWideWaves = 4;            // wavefronts (= packed weight tiles) of a tiled-GEMM workgroup
inline int ffn_gemm_tiles1(int d_e) { return (d_e / 16 + kWideWaves - 1) / kWideWaves; }
__device__ __forceinline__ bool ffn_gemm_on(int4 head, int tiles1, int override_min) {
    return head.y == 64 && head.w > 0 && head.w * tiles1 >= (override_min > 0 ? override_min : kGemmMinWorkgroups);
}
int launch_ffn_wide(const void *X, const void *W13p, const void *W2p, int T, int k, int C, int d_h, int d_e,
                    const int32_t *blocks, const int32_t *perm, const int *ctrl, uint16_t *act_rows,
                    float *Yp, hipStream_t st);

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

__device__ __forceinline__ int lane_id() { return threadIdx.x & (MOE_WAVE - 1); }

__device__ __forceinline__ uint64_t lanemask_lt() {
    return (1ull << lane_id()) - 1ull;
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

}  // namespace moe
