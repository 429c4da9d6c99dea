// C-ABI entry points: host-side validation, argument marshalling, kernel launches.
// Nothing here allocates, copies or synchronises.
#include "dc_internal.h"
#include "advantage_device.h"

namespace dc {

static inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

Workspace carve_workspace(void* base, int32_t n_seq, int64_t dst_capacity_tokens) {
    Workspace w;
    const size_t n = (size_t)(n_seq > 0 ? n_seq : 0);
    w.n_gran = (dst_capacity_tokens > 0 ? (dst_capacity_tokens + GATHER_GRAN - 1) / GATHER_GRAN : 0) + GRAN_TABLE_PAD;
    char* p = static_cast<char*>(base);
    size_t off = 0;
    w.slot_src_off = reinterpret_cast<int64_t*>(p + off); off += round_up(n * sizeof(int64_t), 256);
    w.slot_len = reinterpret_cast<int32_t*>(p + off);     off += round_up(n * sizeof(int32_t), 256);
    w.slot_shard = reinterpret_cast<int32_t*>(p + off);   off += round_up(n * sizeof(int32_t), 256);
    w.gran_first = reinterpret_cast<int32_t*>(p + off);   off += round_up((size_t)w.n_gran * sizeof(int32_t), 256);
    w.gran_rec = reinterpret_cast<GranRec*>(p + off);     off += round_up((size_t)w.n_gran * sizeof(GranRec), 256);
    w.plan_ok = reinterpret_cast<int32_t*>(p + off);      off += 256;     // plan_ok, then own_shard_off, in one block
    w.own_shard_off = w.plan_ok + 16;
    static_assert((16 + DC_MAX_SRC_SHARDS + 1) * sizeof(int32_t) <= 256, "both fit the block");
    w.gpre = nullptr; w.word_starts = nullptr; w.word_last = nullptr;
    if (n_seq > DC_MAX_SEQ) {
        const size_t words = n / 32 + 2;
        w.gpre = reinterpret_cast<int64_t*>(p + off);        off += round_up((n + 1) * sizeof(int64_t), 256);
        w.word_starts = reinterpret_cast<int32_t*>(p + off); off += round_up(words * sizeof(int32_t), 256);
        w.word_last = reinterpret_cast<int32_t*>(p + off);   off += round_up(words * sizeof(int32_t), 256);
    }
    w.bytes = off + 256;
    return w;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// max_seq: DC_MAX_SEQ for the calls whose kernels keep all sequences in one workgroup's LDS (dc_balance,
// dc_balance_group_advantage), DC_MAX_SEQ_LARGE for the others.
static dc_status check_params(const dc_params* prm, int32_t max_seq = DC_MAX_SEQ_LARGE) {
    if (!prm) return DC_ERR_INVALID_ARG;
    if (prm->n_seq < 0 || prm->n_shards < 1 || prm->cap < 0 || prm->align_tokens < 1 || prm->reserved != 0)
        return DC_ERR_INVALID_ARG;
    if (prm->token_budget < 1 || prm->token_budget > 0x7FFFFFFFLL) return DC_ERR_INVALID_ARG;
    if (prm->ddof < 0 || !(prm->eps >= 0.0)) return DC_ERR_INVALID_ARG;
    if (prm->n_seq > max_seq || prm->n_shards > DC_MAX_SHARDS) return DC_ERR_UNSUPPORTED_SIZE;
    return DC_OK;
}

static dc_status check_source(const dc_params* prm, const dc_source* src, SourceDesc* out, bool need_offsets = true) {
    if (!src || !src->shard_seq_off || !src->shard_tokens || src->reserved != 0) return DC_ERR_INVALID_ARG;
    if (src->n_src_shards < 1) return DC_ERR_INVALID_ARG;
    if (src->n_src_shards > DC_MAX_SRC_SHARDS) return DC_ERR_UNSUPPORTED_SIZE;
    if (need_offsets && prm->n_seq > 0 && !src->d_src_tok_off) return DC_ERR_INVALID_ARG;
    out->n_src = src->n_src_shards;
    for (int s = 0; s <= DC_MAX_SRC_SHARDS; ++s) out->seq_off[s] = prm->n_seq;
    for (int s = 0; s < DC_MAX_SRC_SHARDS; ++s) out->tokens[s] = 0;
    if (src->shard_seq_off[0] != 0 || src->shard_seq_off[src->n_src_shards] != prm->n_seq) return DC_ERR_INVALID_ARG;
    for (int s = 0; s < src->n_src_shards; ++s) {
        if (src->shard_seq_off[s + 1] < src->shard_seq_off[s] || src->shard_tokens[s] < 0) return DC_ERR_INVALID_ARG;
        out->seq_off[s] = src->shard_seq_off[s];
        out->tokens[s] = src->shard_tokens[s];
    }
    return DC_OK;
}

// Field descriptors as the kernels take them (by value), with every pointer checked.
static dc_status fill_field_table(const dc_field* fields, int32_t n_fields, const SourceDesc& sd,
                                  int64_t dst_capacity_tokens, FieldTable* out) {
    FieldTable& ft = *out;
    ft.n_fields = n_fields;
    ft.n_src = sd.n_src;
    for (int f = 0; f < DC_MAX_FIELDS + 1; ++f) {
        ft.f[f].dst = nullptr; ft.f[f].elem_bytes = 1; ft.f[f].pad = 0;
        for (int s = 0; s < DC_MAX_SRC_SHARDS; ++s) ft.f[f].src[s] = nullptr;
        if (f >= n_fields) continue;
        const dc_field& in = fields[f];
        if (in.reserved != 0 || !in.src_base) return DC_ERR_INVALID_ARG;
        if (in.elem_bytes != 1 && in.elem_bytes != 2 && in.elem_bytes != 4) return DC_ERR_INVALID_ARG;
        if (dst_capacity_tokens > 0 && (!in.d_dst || !aligned16(in.d_dst))) return DC_ERR_INVALID_ARG;
        ft.f[f].dst = static_cast<char*>(in.d_dst);
        ft.f[f].elem_bytes = in.elem_bytes;
        for (int s = 0; s < sd.n_src; ++s) {
            if (sd.tokens[s] > 0 && (!in.src_base[s] || !aligned16(in.src_base[s]))) return DC_ERR_INVALID_ARG;
            ft.f[f].src[s] = static_cast<const char*>(in.src_base[s]);
        }
    }
    return DC_OK;
}

}  // namespace dc

using namespace dc;

extern "C" {

size_t dc_workspace_bytes(const dc_params* prm, int64_t dst_capacity_tokens) {
    if (!prm) return 0;
    return carve_workspace(nullptr, prm->n_seq, dst_capacity_tokens).bytes;
}

// Host-side checks of dc_balance's arguments; *cap_eff gets the per-shard item limit.
static dc_status check_balance(const dc_params* prm, const int32_t* d_seq_len, const int32_t* d_perm,
                               const int32_t* d_shard_seq_off, const int32_t* d_shard_of_seq,
                               const int64_t* d_shard_load, int32_t* cap_eff, int32_t max_seq = DC_MAX_SEQ) {
    dc_status rc = check_params(prm, max_seq);
    if (rc != DC_OK) return rc;
    if (!d_shard_seq_off || !d_shard_load) return DC_ERR_INVALID_ARG;
    if (prm->n_seq > 0 && (!d_seq_len || !d_perm || !d_shard_of_seq)) return DC_ERR_INVALID_ARG;
    if (prm->cap == 0) {
        if (prm->n_seq % prm->n_shards != 0) return DC_ERR_NOT_DIVISIBLE;     // Algorithm 1 needs K to divide N
        *cap_eff = prm->n_seq / prm->n_shards;
    } else {
        if ((int64_t)prm->cap * prm->n_shards < prm->n_seq) return DC_ERR_INVALID_ARG;
        *cap_eff = prm->cap;
    }
    return DC_OK;
}

// Host-side checks of dc_group_advantage's arguments (prm already checked); fills *sd.
static dc_status check_advantage(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                                 const float* d_reward, const int32_t* d_group_off, int32_t n_groups,
                                 const uint8_t* const* mask_src_base, const float* d_adv_seq,
                                 float* const* adv_tok_src_base, SourceDesc* sd) {
    dc_status rc = check_source(prm, src, sd);
    if (rc != DC_OK) return rc;
    if (n_groups < 0 || n_groups > prm->n_seq || !d_group_off) return DC_ERR_INVALID_ARG;
    if (prm->n_seq > 0 && (!d_seq_len || !d_reward || !d_adv_seq)) return DC_ERR_INVALID_ARG;
    if (adv_tok_src_base) {
        if (!mask_src_base) return DC_ERR_INVALID_ARG;
        for (int s = 0; s < src->n_src_shards; ++s) {
            if (src->shard_tokens[s] == 0) continue;
            if (!mask_src_base[s] || !adv_tok_src_base[s]) return DC_ERR_INVALID_ARG;
            if (!aligned16(mask_src_base[s]) || !aligned16(adv_tok_src_base[s])) return DC_ERR_INVALID_ARG;
        }
    }
    return DC_OK;
}

dc_status dc_balance(const dc_params* prm, const int32_t* d_seq_len,
                     int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                     int64_t* d_shard_load, int32_t* d_status, void* hip_stream) {
    int32_t cap_eff;
    dc_status rc = check_balance(prm, d_seq_len, d_perm, d_shard_seq_off, d_shard_of_seq, d_shard_load, &cap_eff);
    if (rc != DC_OK) return rc;
    hipError_t e = launch_balance(prm->n_seq, prm->n_shards, cap_eff, d_seq_len, d_perm, d_shard_seq_off,
                                  d_shard_of_seq, d_shard_load, d_status, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DC_OK : DC_ERR_HIP;
}

// Workspace of the balance beyond DC_MAX_SEQ sequences: the sort's two index arrays (one of them holds a word per
// sorted item afterwards), the sorted lengths, and the sort's table of digit counts.
static size_t balance_ws_bytes(int32_t n_seq) {
    if (n_seq <= DC_MAX_SEQ) return 0;
    return 3 * (((size_t)n_seq + 63) & ~(size_t)63) * sizeof(int32_t) + dc::sort_large_table_bytes(n_seq) + 256;
}

size_t dc_balance_workspace_bytes(const dc_params* prm) {
    if (!prm || prm->n_seq < 0 || prm->n_seq > DC_MAX_SEQ_LARGE) return 0;
    return balance_ws_bytes(prm->n_seq);
}

dc_status dc_balance_ws(const dc_params* prm, const int32_t* d_seq_len,
                        int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                        int64_t* d_shard_load, void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream) {
    int32_t cap_eff;
    dc_status rc = check_balance(prm, d_seq_len, d_perm, d_shard_seq_off, d_shard_of_seq, d_shard_load, &cap_eff,
                                 DC_MAX_SEQ_LARGE);
    if (rc != DC_OK) return rc;
    if (prm->n_seq <= DC_MAX_SEQ)
        return dc_balance(prm, d_seq_len, d_perm, d_shard_seq_off, d_shard_of_seq, d_shard_load, d_status, hip_stream);
    if (cap_eff > 65535) return DC_ERR_UNSUPPORTED_SIZE;            // a place inside a partition is kept in 16 bits
    if (!d_ws || (reinterpret_cast<uintptr_t>(d_ws) & 255u)) return DC_ERR_INVALID_ARG;
    if (ws_bytes < balance_ws_bytes(prm->n_seq)) return DC_ERR_WORKSPACE;
    hipError_t e = launch_balance_large(prm->n_seq, prm->n_shards, cap_eff, d_seq_len, d_perm, d_shard_seq_off,
                                        d_shard_of_seq, d_shard_load, d_ws, d_status,
                                        static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DC_OK : DC_ERR_HIP;
}

dc_status dc_group_advantage(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                             const float* d_reward, const int32_t* d_group_off, int32_t n_groups,
                             const uint8_t* const* mask_src_base, float* d_adv_seq,
                             float* const* adv_tok_src_base, int32_t* d_status, void* hip_stream) {
    dc_status rc = check_params(prm);
    if (rc != DC_OK) return rc;
    SourceDesc sd;
    rc = check_advantage(prm, src, d_seq_len, d_reward, d_group_off, n_groups, mask_src_base, d_adv_seq,
                         adv_tok_src_base, &sd);
    if (rc != DC_OK) return rc;
    hipError_t e = launch_advantage(prm->n_seq, sd, src->d_src_tok_off, d_seq_len, d_reward, d_group_off, n_groups,
                                    prm->eps, prm->ddof, mask_src_base, d_adv_seq, adv_tok_src_base, d_status,
                                    static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DC_OK : DC_ERR_HIP;
}

dc_status dc_balance_group_advantage(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                                     int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                                     int64_t* d_shard_load, const float* d_reward, const int32_t* d_group_off,
                                     int32_t n_groups, const uint8_t* const* mask_src_base, float* d_adv_seq,
                                     float* const* adv_tok_src_base, int32_t* d_status, void* hip_stream) {
    int32_t cap_eff;
    dc_status rc = check_balance(prm, d_seq_len, d_perm, d_shard_seq_off, d_shard_of_seq, d_shard_load, &cap_eff);
    if (rc != DC_OK) return rc;
    SourceDesc sd;
    rc = check_advantage(prm, src, d_seq_len, d_reward, d_group_off, n_groups, mask_src_base, d_adv_seq,
                         adv_tok_src_base, &sd);
    if (rc != DC_OK) return rc;
    const AdvArgs adv = make_adv_args(prm->n_seq, sd, src->d_src_tok_off, d_seq_len, d_reward, d_group_off, n_groups,
                                      prm->eps, prm->ddof, mask_src_base, d_adv_seq, adv_tok_src_base, d_status);
    hipError_t e = launch_balance_advantage(prm->n_seq, prm->n_shards, cap_eff, d_seq_len, d_perm, d_shard_seq_off,
                                            d_shard_of_seq, d_shard_load, adv, sd, n_groups, d_status,
                                            static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DC_OK : DC_ERR_HIP;
}

dc_status dc_balance_plan_group_advantage(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                                          int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                                          int64_t* d_shard_load, const float* d_reward, const int32_t* d_group_off,
                                          int32_t n_groups, const uint8_t* const* mask_src_base, float* d_adv_seq,
                                          float* const* adv_tok_src_base, int64_t dst_capacity_tokens,
                                          int64_t* d_dst_tok_off, int64_t* d_shard_tok_off, int32_t* d_shard_mb_off,
                                          int32_t* d_mb_seq_off, int32_t* d_cu_seqlens, int32_t* d_n_mb,
                                          void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream) {
    // every argument is checked before anything is enqueued
    int32_t cap_eff;
    dc_status rc = check_balance(prm, d_seq_len, d_perm, d_shard_seq_off, d_shard_of_seq, d_shard_load, &cap_eff);
    if (rc != DC_OK) return rc;
    SourceDesc sd;
    rc = check_advantage(prm, src, d_seq_len, d_reward, d_group_off, n_groups, mask_src_base, d_adv_seq,
                         adv_tok_src_base, &sd);
    if (rc != DC_OK) return rc;
    if (dst_capacity_tokens < 0) return DC_ERR_INVALID_ARG;
    if (!d_dst_tok_off || !d_shard_tok_off || !d_shard_mb_off || !d_mb_seq_off || !d_n_mb || !d_ws) return DC_ERR_INVALID_ARG;
    if (prm->n_seq > 0 && !d_cu_seqlens) return DC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(d_ws) & 255u) return DC_ERR_INVALID_ARG;
    Workspace ws = carve_workspace(d_ws, prm->n_seq, dst_capacity_tokens);
    if (ws_bytes < ws.bytes) return DC_ERR_WORKSPACE;
    if (ws.n_gran > 0x7FFFFFFFLL) return DC_ERR_UNSUPPORTED_SIZE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // the printed algorithm on up to 32 or on 64 workers: the plan runs as the tail of the balance workgroup
    const bool one_launch = prm->n_seq > 0 && (prm->n_shards <= 32 || prm->n_shards == 64) &&
                            (int64_t)cap_eff * prm->n_shards == prm->n_seq;
    if (!one_launch) {
        rc = dc_balance_group_advantage(prm, src, d_seq_len, d_perm, d_shard_seq_off, d_shard_of_seq, d_shard_load, d_reward,
                                        d_group_off, n_groups, mask_src_base, d_adv_seq, adv_tok_src_base, d_status, hip_stream);
        if (rc != DC_OK) return rc;
        return dc_plan(prm, src, d_seq_len, d_perm, d_shard_seq_off, dst_capacity_tokens, d_dst_tok_off, d_shard_tok_off,
                       d_shard_mb_off, d_mb_seq_off, d_cu_seqlens, d_n_mb, d_ws, ws_bytes, d_status, hip_stream);
    }
    const AdvArgs adv = make_adv_args(prm->n_seq, sd, src->d_src_tok_off, d_seq_len, d_reward, d_group_off, n_groups,
                                      prm->eps, prm->ddof, mask_src_base, d_adv_seq, adv_tok_src_base, d_status);
    const PlanArgs plan = make_plan_args(*prm, src->d_src_tok_off, d_seq_len, d_perm, d_shard_seq_off, dst_capacity_tokens,
                                         d_dst_tok_off, d_shard_tok_off, d_shard_mb_off, d_mb_seq_off, d_cu_seqlens, d_n_mb,
                                         ws, d_status);
    hipError_t e = launch_balance_plan_advantage(prm->n_seq, prm->n_shards, cap_eff, d_seq_len, d_perm, d_shard_seq_off,
                                                 d_shard_of_seq, d_shard_load, plan, adv, sd, n_groups, d_status, st);
    if (e != hipSuccess) return DC_ERR_HIP;
    e = launch_records_slots(plan, sd, ws, st);
    return e == hipSuccess ? DC_OK : DC_ERR_HIP;
}

dc_status dc_gae(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len, const float* d_reward,
                 const float* const* value_src_base, const uint8_t* const* mask_src_base,
                 const float* const* logp_src_base, const float* const* ref_logp_src_base,
                 double gamma, double lambda, double kl_coef,
                 float* const* adv_tok_src_base, float* const* ret_tok_src_base,
                 int32_t* d_status, void* hip_stream) {
    dc_status rc = check_params(prm);
    if (rc != DC_OK) return rc;
    SourceDesc sd;
    rc = check_source(prm, src, &sd);
    if (rc != DC_OK) return rc;
    if (!(gamma == gamma) || !(lambda == lambda) || !(kl_coef == kl_coef)) return DC_ERR_INVALID_ARG;   // NaN
    if (!value_src_base || !mask_src_base || !adv_tok_src_base || !ret_tok_src_base) return DC_ERR_INVALID_ARG;
    if (kl_coef != 0.0 && (!logp_src_base || !ref_logp_src_base)) return DC_ERR_INVALID_ARG;
    if (prm->n_seq > 0 && (!d_seq_len || !d_reward)) return DC_ERR_INVALID_ARG;
    for (int s = 0; s < src->n_src_shards; ++s) {
        if (src->shard_tokens[s] == 0) continue;
        const void* need[6] = {value_src_base[s], mask_src_base[s], adv_tok_src_base[s], ret_tok_src_base[s],
                               kl_coef != 0.0 ? logp_src_base[s] : value_src_base[s],
                               kl_coef != 0.0 ? ref_logp_src_base[s] : value_src_base[s]};
        for (const void* p : need)
            if (!p || !aligned16(p)) return DC_ERR_INVALID_ARG;
    }
    hipError_t e = launch_gae(prm->n_seq, sd, src->d_src_tok_off, d_seq_len, d_reward, value_src_base, mask_src_base,
                              logp_src_base, ref_logp_src_base, gamma, lambda, kl_coef, adv_tok_src_base,
                              ret_tok_src_base, d_status, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DC_OK : DC_ERR_HIP;
}

dc_status dc_plan(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                  const int32_t* d_perm, const int32_t* d_shard_seq_off, int64_t dst_capacity_tokens,
                  int64_t* d_dst_tok_off, int64_t* d_shard_tok_off, int32_t* d_shard_mb_off,
                  int32_t* d_mb_seq_off, int32_t* d_cu_seqlens, int32_t* d_n_mb,
                  void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream) {
    dc_status rc = check_params(prm);
    if (rc != DC_OK) return rc;
    SourceDesc sd;
    rc = check_source(prm, src, &sd);
    if (rc != DC_OK) return rc;
    if (dst_capacity_tokens < 0) return DC_ERR_INVALID_ARG;
    if (!d_dst_tok_off || !d_shard_tok_off || !d_shard_mb_off || !d_mb_seq_off || !d_n_mb || !d_ws)
        return DC_ERR_INVALID_ARG;
    if (prm->n_seq > 0 && (!d_seq_len || !d_cu_seqlens)) return DC_ERR_INVALID_ARG;
    // no shard table: the layout is kept, shard for shard (needs no permutation either)
    if (!d_shard_seq_off && (d_perm || prm->n_shards != src->n_src_shards)) return DC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(d_ws) & 255u) return DC_ERR_INVALID_ARG;
    Workspace ws = carve_workspace(d_ws, prm->n_seq, dst_capacity_tokens);
    if (ws_bytes < ws.bytes) return DC_ERR_WORKSPACE;
    if (ws.n_gran > 0x7FFFFFFFLL) return DC_ERR_UNSUPPORTED_SIZE;
    hipError_t e = launch_plan(*prm, sd, src->d_src_tok_off, d_seq_len, d_perm, d_shard_seq_off, dst_capacity_tokens,
                               d_dst_tok_off, d_shard_tok_off, d_shard_mb_off, d_mb_seq_off, d_cu_seqlens, d_n_mb,
                               ws, d_status, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DC_OK : DC_ERR_HIP;
}

dc_status dc_gather(const dc_params* prm, const dc_source* src, const dc_field* fields, int32_t n_fields,
                    int64_t dst_capacity_tokens, const int64_t* d_dst_tok_off,
                    const void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream) {
    return dc_gather_timed(prm, src, fields, n_fields, dst_capacity_tokens, d_dst_tok_off, d_ws, ws_bytes, d_status,
                           hip_stream, nullptr, nullptr);
}

dc_status dc_gather_timed(const dc_params* prm, const dc_source* src, const dc_field* fields, int32_t n_fields,
                          int64_t dst_capacity_tokens, const int64_t* d_dst_tok_off,
                          const void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream,
                          void* hip_event_begins, void* hip_event_ends) {
    (void)d_status;
    dc_status rc = check_params(prm);
    if (rc != DC_OK) return rc;
    SourceDesc sd;
    rc = check_source(prm, src, &sd);
    if (rc != DC_OK) return rc;
    if (n_fields < 0 || dst_capacity_tokens < 0 || !d_dst_tok_off || !d_ws) return DC_ERR_INVALID_ARG;
    if (n_fields > DC_MAX_FIELDS) return DC_ERR_UNSUPPORTED_SIZE;
    if (n_fields > 0 && !fields) return DC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(d_ws) & 255u) return DC_ERR_INVALID_ARG;
    Workspace ws = carve_workspace(const_cast<void*>(d_ws), prm->n_seq, dst_capacity_tokens);
    if (ws_bytes < ws.bytes) return DC_ERR_WORKSPACE;
    if (ws.n_gran > 0x7FFFFFFFLL) return DC_ERR_UNSUPPORTED_SIZE;
    FieldTable ft;
    rc = fill_field_table(fields, n_fields, sd, dst_capacity_tokens, &ft);
    if (rc != DC_OK) return rc;
    hipError_t e = launch_gather(prm->n_seq, ft, dst_capacity_tokens, d_dst_tok_off, ws,
                                 static_cast<hipStream_t>(hip_stream), static_cast<hipEvent_t>(hip_event_begins),
                                 static_cast<hipEvent_t>(hip_event_ends));
    return e == hipSuccess ? DC_OK : DC_ERR_HIP;
}

dc_status dc_gather_advantage(const dc_params* prm, const dc_source* src, const dc_field* fields, int32_t n_fields,
                              int32_t mask_field, const int32_t* d_perm, const float* d_adv_seq, float* d_adv_tok_dst,
                              int64_t dst_capacity_tokens, const int64_t* d_dst_tok_off,
                              const void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream) {
    (void)d_status;
    dc_status rc = check_params(prm);
    if (rc != DC_OK) return rc;
    SourceDesc sd;
    rc = check_source(prm, src, &sd);
    if (rc != DC_OK) return rc;
    if (n_fields < 0 || dst_capacity_tokens < 0 || !d_dst_tok_off || !d_ws) return DC_ERR_INVALID_ARG;
    if (n_fields > DC_MAX_FIELDS) return DC_ERR_UNSUPPORTED_SIZE;
    if (n_fields == 0 || !fields) return DC_ERR_INVALID_ARG;                    // the mask is one of them
    if (mask_field < 0 || mask_field >= n_fields || fields[mask_field].elem_bytes != 1) return DC_ERR_INVALID_ARG;
    if (prm->n_seq > 0 && (!d_perm || !d_adv_seq)) return DC_ERR_INVALID_ARG;
    if (dst_capacity_tokens > 0 && (!d_adv_tok_dst || !aligned16(d_adv_tok_dst))) return DC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(d_ws) & 255u) return DC_ERR_INVALID_ARG;
    Workspace ws = carve_workspace(const_cast<void*>(d_ws), prm->n_seq, dst_capacity_tokens);
    if (ws_bytes < ws.bytes) return DC_ERR_WORKSPACE;
    if (ws.n_gran > 0x7FFFFFFFLL) return DC_ERR_UNSUPPORTED_SIZE;
    FieldTable ft;
    rc = fill_field_table(fields, n_fields, sd, dst_capacity_tokens, &ft);
    if (rc != DC_OK) return rc;
    hipError_t e = launch_gather_advantage(prm->n_seq, ft, mask_field, d_perm, d_adv_seq, d_adv_tok_dst,
                                           dst_capacity_tokens, d_dst_tok_off, ws, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DC_OK : DC_ERR_HIP;
}

dc_status dc_repack(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                    const int32_t* d_perm, const int32_t* d_shard_seq_off,
                    const dc_field* fields, int32_t n_fields, int64_t dst_capacity_tokens,
                    int64_t* d_dst_tok_off, int64_t* d_shard_tok_off, int32_t* d_shard_mb_off,
                    int32_t* d_mb_seq_off, int32_t* d_cu_seqlens, int32_t* d_n_mb,
                    void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream) {
    // validate the gather's arguments before anything is enqueued
    if (n_fields < 0 || (n_fields > 0 && !fields)) return DC_ERR_INVALID_ARG;
    if (n_fields > DC_MAX_FIELDS) return DC_ERR_UNSUPPORTED_SIZE;
    for (int f = 0; f < n_fields; ++f) {
        const dc_field& in = fields[f];
        if (in.reserved != 0 || !in.src_base) return DC_ERR_INVALID_ARG;
        if (in.elem_bytes != 1 && in.elem_bytes != 2 && in.elem_bytes != 4) return DC_ERR_INVALID_ARG;
    }
    dc_status rc = dc_plan(prm, src, d_seq_len, d_perm, d_shard_seq_off, dst_capacity_tokens, d_dst_tok_off,
                           d_shard_tok_off, d_shard_mb_off, d_mb_seq_off, d_cu_seqlens, d_n_mb, d_ws, ws_bytes,
                           d_status, hip_stream);
    if (rc != DC_OK) return rc;
    return dc_gather(prm, src, fields, n_fields, dst_capacity_tokens, d_dst_tok_off, d_ws, ws_bytes, d_status,
                     hip_stream);
}

size_t dc_scatter_workspace_bytes(const dc_params* prm, const dc_source* src) {
    if (!prm || check_params(prm) != DC_OK) return 0;
    SourceDesc sd;
    if (check_source(prm, src, &sd, false) != DC_OK) return 0;
    return carve_scatter_workspace(nullptr, prm->n_seq, sd).bytes;
}

dc_status dc_scatter(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len, const int32_t* d_perm,
                     const dc_field* fields, int32_t n_fields, int64_t dst_capacity_tokens,
                     const int64_t* d_dst_tok_off, void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream) {
    dc_status rc = check_params(prm);
    if (rc != DC_OK) return rc;
    SourceDesc sd;
    rc = check_source(prm, src, &sd);
    if (rc != DC_OK) return rc;
    if (n_fields < 0 || dst_capacity_tokens < 0 || !d_dst_tok_off || !d_ws) return DC_ERR_INVALID_ARG;
    if (prm->n_seq > 0 && (!d_seq_len || !d_perm)) return DC_ERR_INVALID_ARG;
    if (n_fields > DC_MAX_FIELDS) return DC_ERR_UNSUPPORTED_SIZE;
    if (n_fields > 0 && !fields) return DC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(d_ws) & 255u) return DC_ERR_INVALID_ARG;
    ScatterWorkspace ws = carve_scatter_workspace(d_ws, prm->n_seq, sd);
    if (ws_bytes < ws.bytes) return DC_ERR_WORKSPACE;
    FieldTable ft;
    rc = fill_field_table(fields, n_fields, sd, dst_capacity_tokens, &ft);
    if (rc != DC_OK) return rc;
    hipError_t e = launch_scatter(prm->n_seq, sd, src->d_src_tok_off, d_seq_len, d_perm, ft, dst_capacity_tokens,
                                  d_dst_tok_off, ws, d_status, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DC_OK : DC_ERR_HIP;
}

const char* dc_strerror(dc_status code) {
    switch (code) {
        case DC_OK: return "ok";
        case DC_ERR_INVALID_ARG: return "invalid argument";
        case DC_ERR_NOT_DIVISIBLE: return "N mod P != 0 with cap = 0 (Algorithm 1 asserts divisibility)";
        case DC_ERR_UNSUPPORTED_SIZE: return "size above the library's limits";
        case DC_ERR_WORKSPACE: return "workspace too small";
        case DC_ERR_HIP: return "HIP runtime error";
        case DC_ERR_SEQ_EXCEEDS_BUDGET: return "a sequence is longer than the token budget";
        case DC_ERR_ZERO_LENGTH_SEQ: return "a sequence length is <= 0 or above DC_MAX_SEQ_LEN";
        case DC_ERR_OVERFLOW: return "packed layout exceeds the destination capacity";
        case DC_ERR_BAD_LAYOUT: return "inconsistent index data (offsets, groups or permutation)";
    }
    return "unknown status";
}

}  // extern "C"
