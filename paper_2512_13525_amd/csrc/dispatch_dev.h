// Device-side building blocks of a0-a4 (gating selection, Alg. 1, dispatch), shared by the
// stand-alone kernels of moe_route / moe_schedule / moe_permute and by the fused front kernel.
// Each block-level function is written for one workgroup of kFrontThreads threads.
#pragma once

#include "common.h"

namespace moe {

constexpr int kFrontThreads = 1024;
constexpr int kFrontWaves = kFrontThreads / MOE_WAVE;

__device__ __forceinline__ uint64_t readlane_u64(uint64_t v, int l) {
    const uint32_t lo = __builtin_amdgcn_readlane(static_cast<int>(v & 0xffffffffu), l);
    const uint32_t hi = __builtin_amdgcn_readlane(static_cast<int>(v >> 32), l);
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

__device__ __forceinline__ uint64_t readfirstlane_u64(uint64_t v) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<int>(v & 0xffffffffu));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<int>(v >> 32));
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

// ------------------------------------------------------------------ a0: one token per wavefront
// Largest key of the wavefront, in every lane.  Data-parallel-primitive moves instead of LDS-crossbar
// shuffles (the k selection rounds of a token are a chain of these): two exchanges inside quads, two
// rotations inside rows of 16 lanes, then the row results travel to the last lane through the two
// row broadcasts, and a scalar lane read hands the result to everybody.  Lanes a move does not
// write read 0, the smallest key.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint64_t dpp_max_step(uint64_t v) {
    const uint32_t lo = __builtin_amdgcn_update_dpp(0, static_cast<int>(v & 0xffffffffu), CTRL, ROW_MASK, 0xf, false);
    const uint32_t hi = __builtin_amdgcn_update_dpp(0, static_cast<int>(v >> 32), CTRL, ROW_MASK, 0xf, false);
    const uint64_t o = (static_cast<uint64_t>(hi) << 32) | lo;
    return o > v ? o : v;
}

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
    v = dpp_max_step<0xB1, 0xf>(v);                      // quad_perm [1,0,3,2]
    v = dpp_max_step<0x4E, 0xf>(v);                      // quad_perm [2,3,0,1]
    v = dpp_max_step<0x124, 0xf>(v);                     // row_ror:4
    v = dpp_max_step<0x128, 0xf>(v);                     // row_ror:8   -> every lane: its row's largest
    v = dpp_max_step<0x142, 0xa>(v);                     // row_bcast:15 into rows 1 and 3
    v = dpp_max_step<0x143, 0xc>(v);                     // row_bcast:31 into rows 2 and 3 -> lane 63: the largest
    return readlane_u64(v, MOE_WAVE - 1);
}

// Inclusive prefix sum over the 64 lanes with the same moves: three shifts of the input and two of
// the partial sums inside rows of 16 lanes (lanes without a source add 0), then the row totals
// through the row broadcasts.
__device__ __forceinline__ int wave_incl_scan_i32(int v) {
    int s = v;
    s += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);    // row_shr:1
    s += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);    // row_shr:2
    s += __builtin_amdgcn_update_dpp(0, v, 0x113, 0xf, 0xf, true);    // row_shr:3
    s += __builtin_amdgcn_update_dpp(0, s, 0x114, 0xf, 0xe, true);    // row_shr:4, lanes 4..15 of a row
    s += __builtin_amdgcn_update_dpp(0, s, 0x118, 0xf, 0xc, true);    // row_shr:8, lanes 8..15 of a row
    s += __builtin_amdgcn_update_dpp(0, s, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    s += __builtin_amdgcn_update_dpp(0, s, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return s;
}

// Sum over the wavefront, in every lane (fixed order: reproducible).
__device__ __forceinline__ float wave_sum_f32(float v) {
#define MOE_DPP_ADD(ctrl, rows)                                                                   \
    v += __uint_as_float(static_cast<uint32_t>(                                                   \
        __builtin_amdgcn_update_dpp(0, static_cast<int>(__float_as_uint(v)), ctrl, rows, 0xf, false)))
    MOE_DPP_ADD(0xB1, 0xf);                              // quad_perm [1,0,3,2]
    MOE_DPP_ADD(0x4E, 0xf);                              // quad_perm [2,3,0,1]
    MOE_DPP_ADD(0x124, 0xf);                             // row_ror:4
    MOE_DPP_ADD(0x128, 0xf);                             // row_ror:8  -> every lane: its row's sum
    MOE_DPP_ADD(0x142, 0xa);                             // row_bcast:15 into rows 1 and 3
    MOE_DPP_ADD(0x143, 0xc);                             // row_bcast:31 into rows 2 and 3 -> lane 63: the sum
#undef MOE_DPP_ADD
    return __uint_as_float(static_cast<uint32_t>(
        __builtin_amdgcn_readlane(static_cast<int>(__float_as_uint(v)), MOE_WAVE - 1)));
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

// Lane l owns experts l, l+64, ...; every logit becomes a 64-bit key (order-preserving float bits
// in the high word, ~id in the low word) so that "largest logit, lower id on ties" is an unsigned
// comparison.  With one key per lane (E <= 64) the top-k are the keys that fewer than k other keys
// exceed (rank counting with scalar lane broadcasts, no shuffles); with more keys per lane the k
// selections are k maxima, each found with a 6-step cross-lane butterfly.
// row_lds: VPL*64 floats private to this wavefront.  ROW_IN_LDS: `row` already is that LDS copy (the
// caller passes the same address twice and has ordered its writes).  COHERENT: results are written with agent-scope
// stores (read by another workgroup of the same launch).
// mark_lds (optional): a bitset in LDS in which the selected experts are raised.
template <int VPL, bool COHERENT, bool ROW_IN_LDS = false>
__device__ __forceinline__ void route_token(const float *row, int E, int k, const moe_route_cfg &cfg,
                                            float *row_lds, int lane, int32_t *ids_out, float *w_out,
                                            uint32_t *mark_lds = nullptr) {
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
        for (int i = 0; i < VPL; ++i)
            if (!ROW_IN_LDS) row_lds[lane + i * MOE_WAVE] = v[i];
        // the row is private to this wave: a wavefront-scope fence orders its LDS writes
        // before the reads below (no block barrier: waves may be on different tokens)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint64_t gkey = 0ull;
        int owner_shift = 0;                             // group g's key sits in lane g << owner_shift
        if (cfg.n_group <= MOE_WAVE / 8) {
            // eight lanes per group: each scans an eighth of the group, then three exchanges inside the
            // eight lanes merge the (largest, second largest) pairs; the two largest values of a group do
            // not depend on the order in which they are found
            owner_shift = 3;
            const int g = lane >> 3, sub = lane & 7;
            float a = -INFINITY, b = -INFINITY;
            if (g < cfg.n_group) {
                for (int j = sub; j < per; j += 8) {
                    const float x = row_lds[g * per + j];
                    if (x > a) { b = a; a = x; }
                    else if (x > b) { b = x; }
                }
            }
#define MOE_TOP2_MERGE(ctrl)                                                                      \
            do {                                                                                  \
                const float a2 = __uint_as_float(static_cast<uint32_t>(__builtin_amdgcn_update_dpp(  \
                    0, static_cast<int>(__float_as_uint(a)), ctrl, 0xf, 0xf, false)));            \
                const float b2 = __uint_as_float(static_cast<uint32_t>(__builtin_amdgcn_update_dpp(  \
                    0, static_cast<int>(__float_as_uint(b)), ctrl, 0xf, 0xf, false)));            \
                const float hi = a2 > a ? a2 : a, lo = a2 > a ? a : a2;                           \
                const float bb = b2 > b ? b2 : b;                                                 \
                a = hi;                                                                           \
                b = bb > lo ? bb : lo;                                                            \
            } while (0)
            MOE_TOP2_MERGE(0xB1);                        // quad_perm [1,0,3,2]
            MOE_TOP2_MERGE(0x4E);                        // quad_perm [2,3,0,1]
            MOE_TOP2_MERGE(0x141);                       // row_half_mirror: the other quad of the eight
#undef MOE_TOP2_MERGE
            if (sub == 0 && g < cfg.n_group) gkey = make_key(sigmoid_f32(a) + sigmoid_f32(b), g);
        } else if (lane < cfg.n_group) {
            float a = -INFINITY, b = -INFINITY;          // a >= b: two largest logits of the group
            for (int j = 0; j < per; ++j) {
                const float x = row_lds[lane * per + j];
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
            if (lane == (g << owner_shift)) gkey = 0ull;
        }
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int e = lane + i * MOE_WAVE;
            if (e < E && !((keep >> (e / per)) & 1ull)) key[i] = 0ull;
        }
        __builtin_amdgcn_wave_barrier();                 // row_lds is reused by this wave's next token
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

    if (VPL == 1) {
        // Rank of every key among all keys of the row (keys are distinct: the id is part of the key):
        // lane j's keys are broadcast one after the other with scalar lane reads and every lane counts
        // the keys greater than its own.  The k keys with rank < k are the selection, already in
        // output order; dropped or padding keys are 0 and never rank below k.
        int rank[VPL];
    #pragma unroll
        for (int i = 0; i < VPL; ++i) rank[i] = 0;
        for (int j = 0; j < MOE_WAVE; ++j) {
    #pragma unroll
            for (int i2 = 0; i2 < VPL; ++i2) {
                const uint64_t other = readlane_u64(key[i2], j);
    #pragma unroll
                for (int i = 0; i < VPL; ++i) rank[i] += other > key[i] ? 1 : 0;
            }
        }
        float vmax = 0.0f;                                   // largest surviving logit (rank 0)
    #pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const uint64_t top = __ballot(rank[i] == 0 && key[i] != 0ull);
            if (top) vmax = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v[i]), __builtin_ctzll(top)));
        }
        float score[VPL];
        float local = 0.0f;
    #pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const bool sel = rank[i] < k && key[i] != 0ull;
            score[i] = sel ? (cfg.mode == MOE_ROUTE_SIGMOID_GROUP ? sigmoid_f32(v[i]) : expf(v[i] - vmax)) : 0.0f;
            local += score[i];
        }
        const float denom_sel = wave_sum_f32(local);
    #pragma unroll
        for (int i = 0; i < VPL; ++i) {
            if (rank[i] < k && key[i] != 0ull) {
                float w;
                if (cfg.mode == MOE_ROUTE_SIGMOID_GROUP) w = score[i] / denom_sel * cfg.scale;
                else if (cfg.renormalize) w = score[i] / denom_sel;
                else w = score[i] / denom_all;
                const int e = lane + i * MOE_WAVE;
                if (COHERENT) {
                    __hip_atomic_store(ids_out + rank[i], e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    ids_out[rank[i]] = e;
                }
                if (mark_lds) atomicOr(mark_lds + (e >> 5), 1u << (e & 31));
                w_out[rank[i]] = w;
            }
        }
    } else {
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
            if (COHERENT) {
                __hip_atomic_store(ids_out + lane, sel_id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                ids_out[lane] = sel_id;
            }
            if (mark_lds) atomicOr(mark_lds + (sel_id >> 5), 1u << (sel_id & 31));
            w_out[lane] = w;
        }
    }
}

// ------------------------------------------------------------------ a1-a3: Alg. 1 in one workgroup
struct SchedTables {
    const uint64_t *host_mask;     // [E]
    const int16_t  *slot_of;       // [E*n_inst]
    const int32_t  *single_rid;    // [E]
    const uint64_t *multi_mask;    // [n_words]
    const uint64_t *single_mask;   // [n_inst*n_words]
};

struct SchedShared {
    uint32_t flag[MOE_MAX_EXPERTS];
    int32_t rep[MOE_MAX_EXPERTS];
    uint64_t host_mask[MOE_MAX_EXPERTS];
    int32_t single_rid[MOE_MAX_EXPERTS];
    uint64_t multi_mask[MOE_MAX_EXPERTS / 64];
    uint64_t single_mask[MOE_MAX_INSTANCES * (MOE_MAX_EXPERTS / 64)];
};

// 16-byte agent-scope (L2-coherent across XCDs) load of four request ids
__device__ __forceinline__ int4 load_ids4(const int4 *p, bool coherent) {
    if (coherent) {
        int4 v;
        asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
        return v;
    }
    return *p;
}

__device__ __forceinline__ int load_id(const int32_t *p, bool coherent) {
    return coherent ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *p;
}

// One workgroup runs the whole algorithm, so the three steps need no grid-wide synchronisation
// and the schedule is a pure function of (layout, activated set):
//   Step 1 (collect)  every thread scans a strided share of the request ids and raises a flag per
//                     expert in LDS (all writers store the same value);
//   Step 2 (select)   one wavefront turns the flags into 64-bit ballots.  Loads of single-replica
//                     experts are popcounts of (ballot & per-instance mask); lane g holds load[g]
//                     in a register.  Multi-replica experts are walked in ascending id by peeling
//                     bits off (ballot & multi-replica mask); the arg-min over the expert's hosts
//                     reads the candidate lanes' loads with scalar-indexed lane reads, so one greedy
//                     step costs a few scalar instructions per host;
//   Step 3 (rewrite)  every thread maps its share of requests through actRep held in LDS.
// The layout tables are staged into LDS first.  ids_coherent: the ids were written by other
// workgroups of the same launch.  rid and act_rep may be null (the batched launch of the a_max
// study only wants the loads): Step 3 and the actRep stores are then skipped.
// The layout tables into LDS, expert flags cleared (all threads; ends with a barrier).
__device__ __forceinline__ void aebs_stage_tables(const SchedTables &tb, SchedShared &sh, int E, int n_inst, int n_words) {
    const int tid = threadIdx.x;
    for (int e = tid; e < E; e += kFrontThreads) {
        sh.flag[e] = 0u;
        sh.host_mask[e] = tb.host_mask[e];
        sh.single_rid[e] = tb.single_rid[e];
    }
    for (int i = tid; i < n_words; i += kFrontThreads) sh.multi_mask[i] = tb.multi_mask[i];
    for (int i = tid; i < n_inst * n_words; i += kFrontThreads) sh.single_mask[i] = tb.single_mask[i];
    __syncthreads();
}

// Step 2 of Alg. 1 from the expert flags in LDS (first wavefront; the caller orders the flags before
// and sh.rep after with barriers): actRep into sh.rep and act_rep (if not null), loads into load_out.
__device__ __forceinline__ void aebs_select(const SchedTables &tb, SchedShared &sh, int E, int n_inst, int C, int n_words,
                                            int32_t *__restrict__ act_rep, int32_t *__restrict__ load_out) {
    const int tid = threadIdx.x;
    if (tid < MOE_WAVE) {
        const int lane = tid;
        int load = 0;                                   // lane g: load[g]
        for (int w = 0; w < n_words; ++w) {
            const int e = w * 64 + lane;
            const uint64_t act = __ballot(e < E && sh.flag[e] != 0u);
            if (lane < n_inst) load += __popcll(act & sh.single_mask[lane * n_words + w]);
        }
        for (int w = 0; w < n_words; ++w) {
            const int e = w * 64 + lane;
            const uint64_t act = __ballot(e < E && sh.flag[e] != 0u);
            const uint64_t hm = e < E ? sh.host_mask[e] : 0ull;
            uint64_t todo = act & readfirstlane_u64(sh.multi_mask[w]);   // wave-uniform: keep the loop scalar
            int chosen = -1;                            // lane b: instance chosen for expert w*64+b
            while (todo) {
                const int b = __builtin_ctzll(todo);
                todo &= todo - 1;
                uint64_t hosts = readlane_u64(hm, b);
                int best_g = __builtin_ctzll(hosts);
                int best_load = __builtin_amdgcn_readlane(load, best_g);
                hosts &= hosts - 1;
                while (hosts) {                         // ascending instance id: strict '<' keeps the lowest on ties
                    const int h = __builtin_ctzll(hosts);
                    hosts &= hosts - 1;
                    const int l = __builtin_amdgcn_readlane(load, h);
                    if (l < best_load) { best_load = l; best_g = h; }
                }
                if (lane == best_g) load += 1;
                if (lane == b) chosen = best_g;
            }
            if (e < E) {
                int rep = -1;
                if ((act >> lane) & 1ull) {
                    if (chosen >= 0) rep = chosen * C + tb.slot_of[e * n_inst + chosen];
                    else rep = sh.single_rid[e];
                }
                sh.rep[e] = rep;
                if (act_rep) act_rep[e] = rep;
            }
        }
        if (lane < n_inst) load_out[lane] = load;
    }
}

__device__ __forceinline__ void aebs_block(const SchedTables &tb, SchedShared &sh, int E, int n_inst, int C,
                                           int n_words, const int32_t *__restrict__ ids, int n_pairs, int vec_ok,
                                           bool ids_coherent, int32_t *__restrict__ rid,
                                           int32_t *__restrict__ act_rep, int32_t *__restrict__ load_out) {
    const int tid = threadIdx.x;
    aebs_stage_tables(tb, sh, E, n_inst, n_words);

    // ---- Step 1: collect the activated experts
    if (vec_ok) {
        const int n4 = n_pairs >> 2;
        const int4 *ids4 = reinterpret_cast<const int4 *>(ids);
        for (int i = tid; i < n4; i += kFrontThreads) {
            const int4 v = load_ids4(ids4 + i, ids_coherent);
            sh.flag[v.x] = 1u; sh.flag[v.y] = 1u; sh.flag[v.z] = 1u; sh.flag[v.w] = 1u;
        }
        for (int i = (n4 << 2) + tid; i < n_pairs; i += kFrontThreads) sh.flag[load_id(ids + i, ids_coherent)] = 1u;
    } else {
        for (int i = tid; i < n_pairs; i += kFrontThreads) sh.flag[load_id(ids + i, ids_coherent)] = 1u;
    }
    __syncthreads();

    // ---- Step 2: select one replica per activated expert (first wavefront)
    aebs_select(tb, sh, E, n_inst, C, n_words, act_rep, load_out);
    if (!rid) return;                                    // uniform: no barrier is skipped by part of the workgroup
    __syncthreads();

    // ---- Step 3: rewrite every request
    if (vec_ok) {
        const int n4 = n_pairs >> 2;
        const int4 *ids4 = reinterpret_cast<const int4 *>(ids);
        int4 *rid4 = reinterpret_cast<int4 *>(rid);
        for (int i = tid; i < n4; i += kFrontThreads) {
            const int4 v = load_ids4(ids4 + i, ids_coherent);
            int4 r;
            r.x = sh.rep[v.x]; r.y = sh.rep[v.y]; r.z = sh.rep[v.z]; r.w = sh.rep[v.w];
            rid4[i] = r;
        }
        for (int i = (n4 << 2) + tid; i < n_pairs; i += kFrontThreads) rid[i] = sh.rep[load_id(ids + i, ids_coherent)];
    } else {
        for (int i = tid; i < n_pairs; i += kFrontThreads) rid[i] = sh.rep[load_id(ids + i, ids_coherent)];
    }
}

// ------------------------------------------------------------------ a4: dispatch in one workgroup
struct PermShared {
    int cnt[kFrontWaves][MOE_MAX_SLOTS];     // pass A: counts; pass B: running bases
    int total[MOE_MAX_SLOTS];
    int off[MOE_MAX_SLOTS + 1];
    int blk_base[MOE_MAX_SLOTS + 1];         // exclusive scan of the slots' block counts
    int n_wide;                              // 64-row blocks of the slots with more than 64 requests
    int n_wide128;                           // 128-row blocks of the same slots
};

// Exclusive scan over slots of the request totals (sh.total -> sh.off, slot_off), and the place of
// every slot's first block in the FFN work list (-> sh.blk_base; sh.blk_base[C] = number of blocks):
// slots with more than kHeavyRows requests come first, slot order within each class.  First
// wavefront, 64 slots per round.
constexpr int kHeavyRows = 16;
__device__ __forceinline__ void scan_slots(PermShared &sh, int C, int block_rows, int32_t *__restrict__ slot_off,
                                           int lane) {
    int carry = 0, hcarry = 0, lcarry = 0, wide = 0, wide128 = 0;
    for (int s0 = 0; s0 < C; s0 += MOE_WAVE) {
        const int s = s0 + lane;
        const int v = s < C ? sh.total[s] : 0;
        const int nb = (v + block_rows - 1) / block_rows;
        wide += v > 64 ? (v + 63) / 64 : 0;
        wide128 += v > 64 ? (v + 127) / 128 : 0;
        const int hb = v > kHeavyRows ? nb : 0, lb = nb - hb;
        const int incl = wave_incl_scan_i32(v), hincl = wave_incl_scan_i32(hb), lincl = wave_incl_scan_i32(lb);
        if (s < C) {
            sh.off[s] = carry + incl - v;
            slot_off[s] = carry + incl - v;
            // light slots are placed relative to the end of the heavy class, added below
            sh.blk_base[s] = hb ? hcarry + hincl - hb : -(lcarry + lincl - lb) - 1;
        }
        carry += __builtin_amdgcn_readlane(incl, MOE_WAVE - 1);
        hcarry += __builtin_amdgcn_readlane(hincl, MOE_WAVE - 1);
        lcarry += __builtin_amdgcn_readlane(lincl, MOE_WAVE - 1);
    }
    for (int s = lane; s < C; s += MOE_WAVE)
        if (sh.blk_base[s] < 0) sh.blk_base[s] = hcarry + (-sh.blk_base[s] - 1);
    wide = __builtin_amdgcn_readlane(wave_incl_scan_i32(wide), MOE_WAVE - 1);
    wide128 = __builtin_amdgcn_readlane(wave_incl_scan_i32(wide128), MOE_WAVE - 1);
    if (lane == 0) {
        sh.n_wide = wide;
        sh.n_wide128 = wide128;
        sh.off[C] = carry;
        slot_off[C] = carry;
        sh.blk_base[C] = hcarry + lcarry;
    }
}

// Work list of the grouped FFN (a5): the local request rows cut into blocks of at most
// block_rows rows of one slot, in the order scan_slots fixed.  Entry 0 = {number of blocks,
// block_rows, number of 64-row blocks of the slots with more than 64 requests, number of 128-row blocks
// of the same slots}; entry 1+j = {slot, first row, end of the slot's rows, first of the slot's rows}.  All threads, after
// scan_slots and a barrier; one thread per slot writes that slot's entries.
__device__ __forceinline__ void list_blocks(const PermShared &sh, int C, int block_rows,
                                            int32_t *__restrict__ blocks) {
    int4 *out = reinterpret_cast<int4 *>(blocks);
    if (threadIdx.x == 0) out[0] = make_int4(sh.blk_base[C], block_rows, sh.n_wide, sh.n_wide128);
    for (int s = threadIdx.x; s < C; s += blockDim.x) {
        const int lo = sh.off[s], hi = sh.off[s + 1];
        int j = sh.blk_base[s];
        for (int r = lo; r < hi; r += block_rows) out[1 + j++] = make_int4(s, r, hi, lo);
    }
}

// A stable counting sort of the local requests by slot.  Each wavefront owns a contiguous range of
// request ids, so "ascending request id inside a slot" follows from (wave order, group order, lane
// order) and never from the arrival order of atomics:
//   pass A  per-(wave, slot) histograms in LDS;
//   scan    per-slot exclusive prefix over waves, then an exclusive scan over slots;
//   pass B  each wave walks its range again; the lanes of a 64-request group that share a slot are
//           found with a ballot, ranked with a popcount of the lower lanes, and written at the
//           wave's running base for that slot.
__device__ __forceinline__ void permute_block(PermShared &sh, const int32_t *__restrict__ rid, int n_pairs,
                                              int g_self, int C, int32_t *__restrict__ slot_count,
                                              int32_t *__restrict__ slot_off, int32_t *__restrict__ perm,
                                              int32_t *__restrict__ pos, int32_t *__restrict__ blocks,
                                              int block_rows) {
    const int tid = threadIdx.x;
    const int wave = tid / MOE_WAVE;
    const int lane = tid % MOE_WAVE;
    for (int i = tid; i < kFrontWaves * MOE_MAX_SLOTS; i += kFrontThreads) (&sh.cnt[0][0])[i] = 0;
    __syncthreads();

    const int n_groups = (n_pairs + MOE_WAVE - 1) / MOE_WAVE;
    const int gpw = (n_groups + kFrontWaves - 1) / kFrontWaves;
    const int g_begin = wave * gpw;
    const int g_end = min(n_groups, g_begin + gpw);
    const int rid_lo = g_self * C;

    // ---- pass A
    for (int grp = g_begin; grp < g_end; ++grp) {
        const int p = grp * MOE_WAVE + lane;
        const int s = (p < n_pairs ? rid[p] : -1) - rid_lo;
        if (p < n_pairs && s >= 0 && s < C) atomicAdd(&sh.cnt[wave][s], 1);
    }
    __syncthreads();

    // ---- per-slot exclusive prefix over waves
    for (int s = tid; s < C; s += kFrontThreads) {
        int run = 0;
#pragma unroll
        for (int w = 0; w < kFrontWaves; ++w) {
            const int c = sh.cnt[w][s];
            sh.cnt[w][s] = run;
            run += c;
        }
        sh.total[s] = run;
        slot_count[s] = run;
    }
    __syncthreads();

    // ---- exclusive scan over slots, then the FFN's work list
    if (wave == 0) scan_slots(sh, C, block_rows, slot_off, lane);
    __syncthreads();
    list_blocks(sh, C, block_rows, blocks);

    // ---- pass B
    volatile int *base = &sh.cnt[wave][0];
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
            const int b = base[s0] + sh.off[s0];
            if (local && s == s0) row = b + __popcll(same & lanemask_lt());
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

// The same sort cut into chunks of requests, one workgroup per chunk, for batches too large for one
// workgroup (two launches: the grid is the only synchronisation).  hist [n_chunks][C]: requests of
// every chunk per slot.
//   count_chunk    Step 3 of Alg. 1 for the chunk's requests (rid = actRep[id], act_rep staged in
//                  LDS by the caller) and the chunk's row of hist;
//   scatter_chunk  every workgroup rebuilds the slot totals and its own base per slot from hist
//                  (the chunks before it come first inside a slot), then sorts its chunk exactly
//                  like permute_block; the first workgroup also writes the counts, the offsets and
//                  the FFN's work list.
__device__ __forceinline__ void count_chunk(PermShared &sh, const int32_t *__restrict__ rep_lds,
                                            const int32_t *__restrict__ ids, int32_t *__restrict__ rid, int p0, int p1,
                                            int g_self, int C, int32_t *__restrict__ hist_row) {
    const int tid = threadIdx.x;
    for (int s = tid; s < C; s += kFrontThreads) sh.total[s] = 0;
    __syncthreads();
    const int rid_lo = g_self * C;
    for (int p = p0 + tid; p < p1; p += kFrontThreads) {
        const int r = rep_lds[ids[p]];
        rid[p] = r;
        const int s = r - rid_lo;
        if (s >= 0 && s < C) atomicAdd(&sh.total[s], 1);
    }
    __syncthreads();
    for (int s = tid; s < C; s += kFrontThreads) hist_row[s] = sh.total[s];
}

__device__ __forceinline__ void scatter_chunk(PermShared &sh, int *__restrict__ lower, const int32_t *__restrict__ rid,
                                              int p0, int p1, int chunk, int n_chunks, const int32_t *__restrict__ hist,
                                              int g_self, int C, int32_t *__restrict__ slot_count,
                                              int32_t *__restrict__ slot_off, int32_t *__restrict__ perm,
                                              int32_t *__restrict__ pos, int32_t *__restrict__ blocks, int block_rows) {
    const int tid = threadIdx.x;
    const int wave = tid / MOE_WAVE;
    const int lane = tid % MOE_WAVE;
    for (int i = tid; i < kFrontWaves * MOE_MAX_SLOTS; i += kFrontThreads) (&sh.cnt[0][0])[i] = 0;
    // slot totals over all chunks, and the requests of the chunks before this one
    for (int s = tid; s < C; s += kFrontThreads) {
        int tot = 0, low = 0;
        for (int c = 0; c < n_chunks; ++c) {
            const int v = hist[c * C + s];
            tot += v;
            low += c < chunk ? v : 0;
        }
        sh.total[s] = tot;
        lower[s] = low;
        if (chunk == 0) slot_count[s] = tot;
    }
    __syncthreads();

    const int n = p1 - p0;
    const int n_groups = (n + MOE_WAVE - 1) / MOE_WAVE;
    const int gpw = (n_groups + kFrontWaves - 1) / kFrontWaves;
    const int g_begin = wave * gpw;
    const int g_end = min(n_groups, g_begin + gpw);
    const int rid_lo = g_self * C;
    // pass A of the chunk
    for (int grp = g_begin; grp < g_end; ++grp) {
        const int p = p0 + grp * MOE_WAVE + lane;
        const int s = (p < p1 ? rid[p] : -1) - rid_lo;
        if (p < p1 && s >= 0 && s < C) atomicAdd(&sh.cnt[wave][s], 1);
    }
    __syncthreads();
    for (int s = tid; s < C; s += kFrontThreads) {
        int run = 0;
#pragma unroll
        for (int w = 0; w < kFrontWaves; ++w) {
            const int c = sh.cnt[w][s];
            sh.cnt[w][s] = run;
            run += c;
        }
    }
    __syncthreads();
    // offsets of the slots (every workgroup computes them; they are identical) and, once, the work list
    __shared__ int32_t off_sink[MOE_MAX_SLOTS + 1];
    if (wave == 0) scan_slots(sh, C, block_rows, chunk == 0 ? slot_off : off_sink, lane);
    __syncthreads();
    if (chunk == 0) list_blocks(sh, C, block_rows, blocks);

    // pass B of the chunk
    volatile int *base = &sh.cnt[wave][0];
    for (int grp = g_begin; grp < g_end; ++grp) {
        const int p = p0 + grp * MOE_WAVE + lane;
        const int s = (p < p1 ? rid[p] : -1) - rid_lo;
        const bool local = p < p1 && s >= 0 && s < C;
        int row = -1;
        uint64_t todo = __ballot(local);
        while (todo) {
            const int lead = __builtin_ctzll(todo);
            const int s0 = __builtin_amdgcn_readlane(s, lead);
            const uint64_t same = __ballot(local && s == s0);
            const int b = base[s0] + sh.off[s0] + lower[s0];
            if (local && s == s0) row = b + __popcll(same & lanemask_lt());
            __builtin_amdgcn_wave_barrier();
            if (lane == lead) base[s0] += __popcll(same);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            todo &= ~same;
        }
        if (p < p1) {
            pos[p] = row;
            if (local) perm[row] = p;
        }
    }
}

}  // namespace moe
