// Replica layout object: validation on the host and the small device tables the
// scheduler kernel reads (Janus Sec. 3.4, inputs R(e), G(e), P(e,g) of Alg. 1).
#include <stdlib.h>
#include <string.h>

#include <string>
#include <vector>

#include "common.h"

namespace {
thread_local std::string g_last_error;
}

namespace moe {
void set_hip_error(hipError_t e, const char *where) {
    g_last_error = std::string(where) + ": " + hipGetErrorName(e) + " (" + hipGetErrorString(e) + ")";
}
}  // namespace moe

extern "C" const char *moe_strerror(int code) {
    switch (code) {
        case MOE_OK: return "success";
        case MOE_EINVAL: return "invalid argument (null or misaligned pointer, non-positive or inconsistent size)";
        case MOE_ESHAPE: return "unsupported shape";
        case MOE_EPLACEMENT: return "invalid replica layout";
        case MOE_EHIP: return "HIP runtime error (see moe_last_error)";
        case MOE_ENOMEM: return "out of memory";
        case MOE_EWORKSPACE: return "workspace too small";
        default: return "unknown error code";
    }
}

extern "C" const char *moe_last_error(void) { return g_last_error.c_str(); }

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

extern "C" int moe_placement_create(moe_placement_t **out, int E, int n_inst, int C,
                                    const int32_t *slot_to_expert_host) {
    if (!out || !slot_to_expert_host) return MOE_EINVAL;
    *out = nullptr;
    if (E < 1 || n_inst < 1 || C < 1) return MOE_EINVAL;
    if (E > MOE_MAX_EXPERTS || n_inst > MOE_MAX_INSTANCES || C > MOE_MAX_SLOTS) return MOE_ESHAPE;

    const int S = n_inst * C;
    const int n_words = (E + 63) / 64;
    std::vector<uint64_t> host_mask(E, 0);
    std::vector<int16_t> slot_of(static_cast<size_t>(E) * n_inst, -1);
    std::vector<int32_t> R(E, 0);
    for (int g = 0; g < n_inst; ++g) {
        for (int s = 0; s < C; ++s) {
            const int32_t e = slot_to_expert_host[g * C + s];
            if (e == -1) continue;
            if (e < 0 || e >= E) return MOE_EPLACEMENT;
            if (host_mask[e] & (1ull << g)) return MOE_EPLACEMENT;   // two replicas on one instance
            host_mask[e] |= 1ull << g;
            slot_of[static_cast<size_t>(e) * n_inst + g] = static_cast<int16_t>(s);
            R[e] += 1;
        }
    }
    for (int e = 0; e < E; ++e)
        if (R[e] == 0) return MOE_EPLACEMENT;

    std::vector<int32_t> single_rid(E, -1);
    std::vector<uint64_t> multi_mask(n_words, 0);
    std::vector<uint64_t> single_mask(static_cast<size_t>(n_inst) * n_words, 0);
    for (int e = 0; e < E; ++e) {
        if (R[e] == 1) {
            const int g = __builtin_ctzll(host_mask[e]);
            single_rid[e] = g * C + slot_of[static_cast<size_t>(e) * n_inst + g];
            single_mask[static_cast<size_t>(g) * n_words + e / 64] |= 1ull << (e % 64);
        } else {
            multi_mask[e / 64] |= 1ull << (e % 64);
        }
    }

    moe_placement *pl = static_cast<moe_placement *>(calloc(1, sizeof(moe_placement)));
    if (!pl) return MOE_ENOMEM;
    pl->E = E; pl->n_inst = n_inst; pl->C = C; pl->n_words = n_words;
    pl->slot_to_expert_h = static_cast<int32_t *>(malloc(sizeof(int32_t) * S));
    pl->R_h = static_cast<int32_t *>(malloc(sizeof(int32_t) * E));
    if (!pl->slot_to_expert_h || !pl->R_h) { moe_placement_destroy(pl); return MOE_ENOMEM; }
    memcpy(pl->slot_to_expert_h, slot_to_expert_host, sizeof(int32_t) * S);
    memcpy(pl->R_h, R.data(), sizeof(int32_t) * E);

    const size_t o_hm = 0;
    const size_t o_so = align_up(o_hm + sizeof(uint64_t) * E, 256);
    const size_t o_sr = align_up(o_so + sizeof(int16_t) * E * n_inst, 256);
    const size_t o_mm = align_up(o_sr + sizeof(int32_t) * E, 256);
    const size_t o_sm = align_up(o_mm + sizeof(uint64_t) * n_words, 256);
    const size_t total = align_up(o_sm + sizeof(uint64_t) * n_inst * n_words, 256);

    hipError_t err = hipGetDevice(&pl->device);
    if (err == hipSuccess) err = hipMalloc(&pl->dev_block, total);
    if (err != hipSuccess) {
        moe::set_hip_error(err, "moe_placement_create/hipMalloc");
        pl->dev_block = nullptr;
        moe_placement_destroy(pl);
        return err == hipErrorOutOfMemory ? MOE_ENOMEM : MOE_EHIP;
    }
    std::vector<char> stage(total, 0);
    memcpy(stage.data() + o_hm, host_mask.data(), sizeof(uint64_t) * E);
    memcpy(stage.data() + o_so, slot_of.data(), sizeof(int16_t) * E * n_inst);
    memcpy(stage.data() + o_sr, single_rid.data(), sizeof(int32_t) * E);
    memcpy(stage.data() + o_mm, multi_mask.data(), sizeof(uint64_t) * n_words);
    memcpy(stage.data() + o_sm, single_mask.data(), sizeof(uint64_t) * n_inst * n_words);
    err = hipMemcpy(pl->dev_block, stage.data(), total, hipMemcpyHostToDevice);
    if (err != hipSuccess) {
        moe::set_hip_error(err, "moe_placement_create/hipMemcpy");
        moe_placement_destroy(pl);
        return MOE_EHIP;
    }
    char *base = static_cast<char *>(pl->dev_block);
    pl->host_mask_d = reinterpret_cast<uint64_t *>(base + o_hm);
    pl->slot_of_d = reinterpret_cast<int16_t *>(base + o_so);
    pl->single_rid_d = reinterpret_cast<int32_t *>(base + o_sr);
    pl->multi_mask_d = reinterpret_cast<uint64_t *>(base + o_mm);
    pl->single_mask_d = reinterpret_cast<uint64_t *>(base + o_sm);
    *out = pl;
    return MOE_OK;
}

extern "C" void moe_placement_destroy(moe_placement_t *pl) {
    if (!pl) return;
    if (pl->dev_block) {
        (void)hipDeviceSynchronize();
        (void)hipFree(pl->dev_block);
    }
    free(pl->slot_to_expert_h);
    free(pl->R_h);
    free(pl);
}

extern "C" int moe_placement_replicas(const moe_placement_t *pl, int e) {
    if (!pl || e < 0 || e >= pl->E) return MOE_EINVAL;
    return pl->R_h[e];
}

extern "C" int moe_placement_dims(const moe_placement_t *pl, int *E, int *n_inst, int *C) {
    if (!pl) return MOE_EINVAL;
    if (E) *E = pl->E;
    if (n_inst) *n_inst = pl->n_inst;
    if (C) *C = pl->C;
    return MOE_OK;
}
