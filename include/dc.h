/*
 * dc.h - C ABI of the MI355X Data Coordinator reshard path.
 *
 * The path is what the paper's Data Coordinator does when two consecutive RL
 * stages use different data-parallel layouts (Sec. 6, "Distributed Databuffer"
 * and "Load Balancing"; App. B: the advantage -> actor-log-prob transition is
 * the one DP-layout change of a GRPO step):
 *
 *   dc_balance          Algorithm 1, Constrained LPT Load Balancing: N sequence
 *                       lengths -> P shards of (by default) exactly N/P sequences
 *                       (dc_balance_ws: the same for more than DC_MAX_SEQ sequences).
 *   dc_group_advantage  the "advantage" stage of GRPO (Sec. 1 payload list,
 *                       App. B Table 2): each response's reward normalised by
 *                       its prompt group's mean and std, then broadcast over the
 *                       response's loss-bearing tokens, in the rollout layout.
 *   dc_plan             packed training layout of the P shards: token offsets,
 *                       token-budget micro-batches, cu_seqlens.
 *   dc_gather           segmented copy of every per-token field from the rollout
 *                       layout into the packed training layout.
 *   dc_repack           dc_plan followed by dc_gather.
 *   dc_gather_advantage dc_gather that makes the per-token advantage field on the way,
 *                       from the per-sequence advantages and the loss mask.
 *   dc_scatter          the reverse path: per-token fields a training-layout stage
 *                       produced go back from the packed training layout to the
 *                       rollout layout (the collect / concat side of a stage
 *                       transition, App. B Table 2).
 *   dc_gae              the advantage stage of PPO (Sec. 7.1 evaluates PPO with a critic).
 *   dc_balance_group_advantage, dc_balance_plan_group_advantage
 *                       the calls above that depend on nothing but the lengths and the rewards, issued
 *                       as one and as two launches (same results).
 *   dc_repack_noalloc, dc_gather_timed
 *                       dc_repack without a workspace argument, for callers that cannot allocate;
 *                       dc_gather whose dispatch carries the caller's timing events.
 *
 * Conventions
 *   - Pointers named d_* are DEVICE pointers (gfx950, current HIP device).  All
 *     other pointers are HOST pointers, read during the call only.
 *   - The caller owns every buffer: inputs, outputs and workspace.  The library
 *     allocates nothing and keeps no state between calls (dc_repack_noalloc alone
 *     plans in a device array of the library's own, see there).
 *   - Every call only enqueues kernels on `hip_stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and returns; nothing synchronises.
 *   - The return value reports what the host can check without a sync.  Errors
 *     that depend on device data are written by the kernels to *d_status (an
 *     int32 the caller zeroes beforehand; the first error wins; outputs are then
 *     unspecified but no access leaves the caller's buffers).
 *   - Identical inputs give bit-identical outputs on every run.
 *
 * Layouts
 *   Rollout (source) layout: n_src_shards packed buffers per field.  Rollout shard
 *   s holds sequences [shard_seq_off[s], shard_seq_off[s+1]) in index order;
 *   sequence i occupies elements [d_src_tok_off[i], d_src_tok_off[i] + seq_len[i])
 *   of its shard's buffer (offsets restart in every shard, non-overlapping,
 *   increasing with i inside a shard).  A sequence is prompt tokens then response
 *   tokens.  Prompt groups are contiguous runs of sequences, d_group_off is their
 *   CSR offset array.
 *
 *   Training (destination) layout: one arena per field.  Output slot j holds
 *   sequence d_perm[j]; shard p owns slots [d_shard_seq_off[p], d_shard_seq_off[p+1])
 *   and the token range [d_shard_tok_off[p], d_shard_tok_off[p] + load_p);
 *   d_shard_tok_off[p+1] is that end rounded up to align_tokens (padding elements
 *   are never written).  Slot j starts at element d_dst_tok_off[j].
 *   Micro-batch m covers slots [d_mb_seq_off[m], d_mb_seq_off[m+1]), never spans
 *   shards, and is built by next-fit in slot order: a slot joins the open
 *   micro-batch iff its tokens still fit under token_budget.  Its cu_seqlens slice
 *   has n_m + 1 int32 entries starting at index d_mb_seq_off[m] + m: 0, then the
 *   running token totals.  Shard p owns micro-batches
 *   [d_shard_mb_off[p], d_shard_mb_off[p+1]).
 */
#ifndef DC_H
#define DC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DC_MAX_SEQ        16384   /* N of dc_balance, dc_balance_group_advantage: one   */
                                  /*    workgroup sorts and assigns in LDS            */
#define DC_MAX_SEQ_LARGE  1048576 /* N of every other call (dc_balance_ws among them); */
                                  /*    above DC_MAX_SEQ the balance and the plan take  */
                                  /*    slower paths through workspace memory          */
#define DC_MAX_SHARDS     1024    /* P: one lane per shard (one wavefront up to 64,   */
                                  /*    the whole workgroup above)                    */
#define DC_MAX_FIELDS     8
#define DC_MAX_SRC_SHARDS 16
#define DC_MAX_SEQ_LEN    (1 << 24)
#define DC_REPACK_NOALLOC_WS_BYTES (8u << 20)   /* the device array dc_repack_noalloc plans in */

typedef enum dc_status {
    DC_OK = 0,
    DC_ERR_INVALID_ARG = 1,        /* null pointer, bad size, bad alignment, bad index data      */
    DC_ERR_NOT_DIVISIBLE = 2,      /* cap = 0 and N mod P != 0 (Algorithm 1's assertion)         */
    DC_ERR_UNSUPPORTED_SIZE = 3,   /* N, P, field or rollout-shard count above the DC_MAX_* limit*/
    DC_ERR_WORKSPACE = 4,          /* workspace smaller than dc_workspace_bytes()                */
    DC_ERR_HIP = 5,                /* a HIP runtime call failed                                  */
    DC_ERR_SEQ_EXCEEDS_BUDGET = 6, /* device: a sequence is longer than token_budget             */
    DC_ERR_ZERO_LENGTH_SEQ = 7,    /* device: a sequence length is <= 0 (or > DC_MAX_SEQ_LEN)    */
    DC_ERR_OVERFLOW = 8,           /* device: packed layout does not fit dst_capacity_tokens     */
    DC_ERR_BAD_LAYOUT = 9          /* device: rollout offsets out of range / overlapping, group
                                      offsets not monotone, perm not a permutation               */
} dc_status;

typedef struct dc_params {
    int32_t n_seq;          /* N                                                              */
    int32_t n_shards;       /* P  (K of Algorithm 1), 1..DC_MAX_SHARDS                        */
    int32_t cap;            /* 0: C = N/P as in Algorithm 1; >0: per-shard item limit
                               (cap >= N makes the constraint vacuous: textbook LPT)          */
    int32_t align_tokens;   /* >= 1; shard starts are multiples of it (1 = dense)             */
    int64_t token_budget;   /* micro-batch token cap, 1 .. 2^31-1                             */
    double  eps;            /* added to the group std                                         */
    int32_t ddof;           /* 0 population std, 1 Bessel-corrected                           */
    int32_t reserved;       /* must be 0                                                      */
} dc_params;

/* Where the sequences live in the rollout layout. */
typedef struct dc_source {
    int32_t        n_src_shards;   /* 1..DC_MAX_SRC_SHARDS                                    */
    int32_t        reserved;       /* must be 0                                               */
    const int32_t* shard_seq_off;  /* HOST [n_src_shards+1], [0]=0, last=N, non-decreasing    */
    const int64_t* shard_tokens;   /* HOST [n_src_shards], elements each rollout buffer holds */
    const int64_t* d_src_tok_off;  /* DEVICE [N]                                              */
} dc_source;

/* One per-token field.  src_base[s] and dst must be 16-byte aligned device pointers.  The
 * rollout buffers are read in aligned 4-byte words: a buffer of 1- or 2-byte elements must be
 * readable up to the next multiple of 4 bytes past its last element (never written). */
typedef struct dc_field {
    const void* const* src_base;   /* HOST [n_src_shards] device base pointers                */
    void*              d_dst;      /* DEVICE arena of dst_capacity_tokens elements            */
    int32_t            elem_bytes; /* 1, 2 or 4                                               */
    int32_t            reserved;   /* must be 0                                               */
} dc_field;

/* Bytes of device workspace dc_plan / dc_gather / dc_repack need for these sizes
 * (about 70 bytes per 1024 tokens of capacity plus 16 bytes per sequence; above DC_MAX_SEQ
 * sequences 8.25 bytes per sequence more).  The workspace is where the re-partitioning of
 * Sec. 6 "Distributed Databuffer" keeps its routing tables between dc_plan and dc_gather: which
 * sequence of which rollout shard each piece of the training layout comes from.  It is the
 * caller's, like every buffer (the paper's Databuffer owns its storage; here nothing is owned).
 * Returns 0 for a null prm. */
size_t dc_workspace_bytes(const dc_params* prm, int64_t dst_capacity_tokens);

/*
 * Algorithm 1 (Constrained LPT Load Balancing).
 *   I = argsort(d_seq_len, descending), equal lengths in ascending index order;
 *   each u in I goes to the worker with the lexicographically smallest (load, k)
 *   among workers holding fewer than C items; its load grows by the length.
 * Outputs (device): d_perm[N] members of P_0, P_1, ... in insertion order;
 * d_shard_seq_off[P+1]; d_shard_of_seq[N]; d_shard_load[P] (tokens).
 * Host errors: INVALID_ARG, NOT_DIVISIBLE, UNSUPPORTED_SIZE, HIP.
 * Device errors: ZERO_LENGTH_SEQ.
 */
dc_status dc_balance(const dc_params* prm, const int32_t* d_seq_len,
                     int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                     int64_t* d_shard_load, int32_t* d_status, void* hip_stream);

/*
 * dc_balance for up to DC_MAX_SEQ_LARGE sequences (same results, same errors).  Up to DC_MAX_SEQ
 * sequences it is dc_balance itself and d_ws may be NULL.  Above, it is a chain of launches on the stream:
 * the sort of Algorithm 1's first statement runs over many workgroups and keeps its index arrays, the sorted
 * lengths and its digit counts in d_ws (256-byte aligned, dc_balance_workspace_bytes(prm) bytes: about 13 bytes
 * per sequence); the assignment is one workgroup that takes the sorted sequences DC_MAX_SEQ at a time,
 * carrying the workers' loads along; a last launch writes d_perm and d_shard_of_seq.  d_ws holds nothing the
 * caller needs afterwards.  Limit above DC_MAX_SEQ: at most 65535 sequences per shard (C of Algorithm 1, or
 * prm->cap), else UNSUPPORTED_SIZE.
 */
size_t dc_balance_workspace_bytes(const dc_params* prm);
dc_status dc_balance_ws(const dc_params* prm, const int32_t* d_seq_len,
                        int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                        int64_t* d_shard_load, void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream);

/*
 * Group-relative advantage.  For group g with rewards r_1..r_G (float32):
 *   mean = sum r / G,  var = sum (r - mean)^2 / (G - ddof),
 *   A_i = (r_i - mean) / (sqrt(var) + eps), evaluated in float64, stored as float32.
 *   A group with G - ddof <= 0, or whose rewards are all bit-identical, gets +0.
 * d_adv_seq[N] receives A_i.  If adv_tok_src_base != NULL, each rollout shard s also
 * gets its per-token advantages: element t of sequence i is A_i where
 * mask_src_base[s][t] != 0 and +0.0f elsewhere; elements outside every sequence are
 * left untouched.  mask_src_base / adv_tok_src_base: HOST arrays [n_src_shards] of
 * 16-byte aligned device pointers (uint8 / float32 buffers of shard_tokens[s] elements).
 * Device errors: BAD_LAYOUT, ZERO_LENGTH_SEQ.
 */
dc_status dc_group_advantage(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                             const float* d_reward, const int32_t* d_group_off, int32_t n_groups,
                             const uint8_t* const* mask_src_base, float* d_adv_seq,
                             float* const* adv_tok_src_base, int32_t* d_status, void* hip_stream);

/*
 * dc_balance and dc_group_advantage in ONE launch (same arguments, same results, same device errors):
 * the two stages are independent, the balance keeps one compute unit busy for its whole run and the
 * advantage stage streams the tokens meanwhile.  For callers that would otherwise put the two on two
 * streams: this needs no second stream and no cross-stream wait.
 */
dc_status dc_balance_group_advantage(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                                     int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                                     int64_t* d_shard_load, const float* d_reward, const int32_t* d_group_off,
                                     int32_t n_groups, const uint8_t* const* mask_src_base, float* d_adv_seq,
                                     float* const* adv_tok_src_base, int32_t* d_status, void* hip_stream);

/*
 * dc_balance_group_advantage followed by dc_plan, with fewer launches (same arguments as the two calls,
 * same results, same device errors, every argument checked before anything is enqueued): the three
 * steps that come before the data movement in the re-partitioning of Sec. 6 - Algorithm 1 ("Load
 * Balancing"), the advantage stage, and the layout the "Distributed Databuffer" redistributes into.
 * With Algorithm 1 as printed (cap = 0 or cap * P = N) on 1 .. 32 or on 64 shards and up to DC_MAX_SEQ
 * sequences, the plan runs as the tail of the workgroup that balances: that workgroup holds every output
 * slot's sequence and length when it is done, which is all the plan reads.  Two launches instead of
 * five; dc_gather (or dc_gather_advantage) follows as after dc_plan.  Other shapes: the two calls one after
 * the other.
 */
dc_status dc_balance_plan_group_advantage(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                                          int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                                          int64_t* d_shard_load, const float* d_reward, const int32_t* d_group_off,
                                          int32_t n_groups, const uint8_t* const* mask_src_base, float* d_adv_seq,
                                          float* const* adv_tok_src_base, int64_t dst_capacity_tokens,
                                          int64_t* d_dst_tok_off, int64_t* d_shard_tok_off, int32_t* d_shard_mb_off,
                                          int32_t* d_mb_seq_off, int32_t* d_cu_seqlens, int32_t* d_n_mb,
                                          void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream);

/*
 * Generalized advantage estimation (Schulman et al. 2016, arXiv 1506.02438, eqs. 11-16): the
 * advantage stage of PPO (Sec. 7.1 evaluates PPO with a critic; App. B Table 2 "advantage"), per
 * token, in the rollout layout.  With t_1 < ... < t_m the tokens of sequence i whose mask byte is
 * non-zero (tokens without loss are stepped over):
 *   r_k     = -kl_coef * (logp[t_k] - ref_logp[t_k])  + (k == m ? d_reward[i] : 0)
 *   delta_k = r_k + gamma * V[t_{k+1}] - V[t_k],   V[t_{m+1}] = 0
 *   A_k     = delta_k + gamma * lambda * A_{k+1},  A_{m+1} = 0;   ret_k = A_k + V[t_k]
 * evaluated in float64 and rounded once to float32.  adv_tok / ret_tok get A_k / ret_k at t_k and
 * +0.0 at every other token of the sequence; elements that belong to no sequence are left alone.
 * value_src_base[s] (float32), mask_src_base[s] (uint8), adv_tok_src_base[s], ret_tok_src_base[s]
 * (float32, written): host arrays of src->n_src_shards device pointers to 16-byte aligned buffers
 * of src->shard_tokens[s] elements.  logp_src_base / ref_logp_src_base (float32, same shape) are
 * read only when kl_coef != 0 and may be NULL otherwise.
 * Device errors: BAD_LAYOUT, ZERO_LENGTH_SEQ.
 */
dc_status dc_gae(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len, const float* d_reward,
                 const float* const* value_src_base, const uint8_t* const* mask_src_base,
                 const float* const* logp_src_base, const float* const* ref_logp_src_base,
                 double gamma, double lambda, double kl_coef,
                 float* const* adv_tok_src_base, float* const* ret_tok_src_base,
                 int32_t* d_status, void* hip_stream);

/*
 * Plan of the packed training layout (see "Layouts"): where the Databuffer of Sec. 6 ("Distributed
 * Databuffer": redistribution between two stages whose DP sizes differ) puts every sequence once
 * Algorithm 1 has said which worker takes it.  The paper pads its batches (Sec. 7.1); the packed
 * form, the token-budget micro-batches and cu_seqlens follow the statement of the task this library
 * serves, as read under "Layouts" above.
 * d_perm / d_shard_seq_off: as dc_balance wrote them, or any permutation and shard table.
 * d_perm == NULL: no re-partitioning, slot j holds sequence j.  d_shard_seq_off == NULL (then d_perm
 * must be NULL and prm->n_shards == src->n_src_shards, else INVALID_ARG): the training shards ARE the
 * rollout shards.  That is the case of Sec. 6 "Local Cache" - the DP size does not change between the
 * two stages, so the data stays where it is: with packed rollout buffers the plan then describes them
 * in place (d_dst_tok_off[j] - d_shard_tok_off[shard of j] == d_src_tok_off[j]), the next stage reads
 * them through it and no dc_gather is needed.
 * Outputs (device):
 * d_dst_tok_off[N+1] (last = d_shard_tok_off[P]), d_shard_tok_off[P+1], d_shard_mb_off[P+1],
 * d_mb_seq_off[N+1] (first M+1 entries valid), d_cu_seqlens[2N] (first N+M valid), d_n_mb[1] = M.
 * Also fills the workspace with what dc_gather needs.  dst_capacity_tokens is the
 * element count of every destination arena.
 * Device errors: ZERO_LENGTH_SEQ, SEQ_EXCEEDS_BUDGET, OVERFLOW, BAD_LAYOUT.
 */
dc_status dc_plan(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                  const int32_t* d_perm, const int32_t* d_shard_seq_off, int64_t dst_capacity_tokens,
                  int64_t* d_dst_tok_off, int64_t* d_shard_tok_off, int32_t* d_shard_mb_off,
                  int32_t* d_mb_seq_off, int32_t* d_cu_seqlens, int32_t* d_n_mb,
                  void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream);

/*
 * Segmented gather: the data movement of the Databuffer's re-partitioning (Sec. 6 "Distributed
 * Databuffer"; App. B Table 2 counts it as put / get), for the payload fields of Sec. 1 (token ids,
 * masks, log-probs, values, advantages).  For every slot j and field f copy seq_len[perm[j]] elements from
 * the sequence's place in the rollout layout to element d_dst_tok_off[j] of f.d_dst,
 * as raw bytes.  Must follow a dc_plan on the same stream with the same prm, src,
 * dst_capacity_tokens, d_dst_tok_off and workspace.
 */
dc_status dc_gather(const dc_params* prm, const dc_source* src, const dc_field* fields, int32_t n_fields,
                    int64_t dst_capacity_tokens, const int64_t* d_dst_tok_off,
                    const void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream);

/*
 * dc_gather whose kernel dispatch carries two events of the caller (hipEvent_t, created with timing enabled;
 * either may be NULL): hip_event_begins is updated with the time at which the gather kernel starts on the device,
 * hip_event_ends with the time at which it ends, so that hipEventElapsedTime(begins, ends) is the kernel's own
 * duration (what a profiler's kernel trace reports), without the gaps that events recorded before and after the
 * call add.  For callers that measure the data movement of Sec. 6's re-partitioning (Sec. 7 reports its
 * throughput) in place.  Same arguments, results and errors as dc_gather otherwise; with an empty batch (no
 * sequences, fields or capacity) nothing is launched and the events are left as they are.
 */
dc_status dc_gather_timed(const dc_params* prm, const dc_source* src, const dc_field* fields, int32_t n_fields,
                          int64_t dst_capacity_tokens, const int64_t* d_dst_tok_off,
                          const void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream,
                          void* hip_event_begins, void* hip_event_ends);

/*
 * dc_gather that also makes the per-token advantage field (Sec. 1 payload list; App. B Table 2
 * "advantage") directly in the training layout, from the per-sequence advantages:
 *   d_adv_tok_dst[d_dst_tok_off[j] + t] = m != 0 ? d_adv_seq[d_perm[j]] : +0.0f,
 * m = the byte of token t of sequence d_perm[j] in fields[mask_field] (elem_bytes 1, the loss mask).
 * The result is what dc_group_advantage's per-token buffers would give when gathered as one more
 * float32 field, without those buffers: call dc_group_advantage (or dc_balance_group_advantage) with
 * adv_tok_src_base = NULL before.  The gather then reads 1 byte per token where it would read 4,
 * and the advantage stage writes no per-token data.
 * d_adv_tok_dst: 16-byte aligned float32 arena of dst_capacity_tokens elements (padding elements are
 * never written).  d_perm[N], d_adv_seq[N]: as dc_balance / dc_group_advantage left them; the plan
 * in the workspace must come from the same d_perm.  Everything else as for dc_gather.
 */
dc_status dc_gather_advantage(const dc_params* prm, const dc_source* src, const dc_field* fields, int32_t n_fields,
                              int32_t mask_field, const int32_t* d_perm, const float* d_adv_seq, float* d_adv_tok_dst,
                              int64_t dst_capacity_tokens, const int64_t* d_dst_tok_off,
                              const void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream);

/* dc_plan then dc_gather: the whole re-partitioning of Sec. 6 "Distributed Databuffer" for one
 * batch, once dc_balance (Sec. 6 "Load Balancing") has assigned the sequences.  Arguments, errors
 * and NULL conventions are those of the two calls; the gather's arguments are checked before the
 * plan is enqueued. */
dc_status dc_repack(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                    const int32_t* d_perm, const int32_t* d_shard_seq_off,
                    const dc_field* fields, int32_t n_fields, int64_t dst_capacity_tokens,
                    int64_t* d_dst_tok_off, int64_t* d_shard_tok_off, int32_t* d_shard_mb_off,
                    int32_t* d_mb_seq_off, int32_t* d_cu_seqlens, int32_t* d_n_mb,
                    void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream);

/*
 * dc_repack without a workspace argument, for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The plan's
 * workspace is a device array of DC_REPACK_NOALLOC_WS_BYTES (8 MiB) inside the library; each GPU the
 * library runs on holds its own copy until the process ends.  The call allocates and frees
 * nothing.  Arguments, results, host and device errors are dc_repack's; the device that owns the
 * buffers and the stream must be the current HIP device.
 * Limit: dc_workspace_bytes(prm, dst_capacity_tokens) must not exceed DC_REPACK_NOALLOC_WS_BYTES
 * (about 120 M tokens of capacity with 16 384 sequences), else UNSUPPORTED_SIZE and nothing is
 * enqueued.
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap there (two
 * streams, two threads) race; calls on one stream do not.  A dc_gather / dc_scatter that is to
 * reuse the plan later needs dc_repack with a workspace of the caller's.
 */
dc_status dc_repack_noalloc(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                            const int32_t* d_perm, const int32_t* d_shard_seq_off,
                            const dc_field* fields, int32_t n_fields, int64_t dst_capacity_tokens,
                            int64_t* d_dst_tok_off, int64_t* d_shard_tok_off, int32_t* d_shard_mb_off,
                            int32_t* d_mb_seq_off, int32_t* d_cu_seqlens, int32_t* d_n_mb,
                            int32_t* d_status, void* hip_stream);

/* Bytes of device workspace dc_scatter needs (256-byte aligned, like dc_plan's). */
size_t dc_scatter_workspace_bytes(const dc_params* prm, const dc_source* src);

/*
 * Reverse of dc_gather.  For every slot j and field f, seq_len[perm[j]] elements go from element
 * d_dst_tok_off[j] of the field's training arena to the sequence's place in its rollout buffer, as
 * raw bytes.  In each dc_field the roles are swapped: d_dst is the training arena (READ, 16-byte
 * aligned, dst_capacity_tokens elements, readable in whole 4-byte words) and src_base[s] are the
 * rollout buffers (WRITTEN, 16-byte aligned).  Elements of a rollout buffer that belong to no sequence
 * (padding between rows) are left untouched.  d_dst_tok_off: as dc_plan wrote it for the same prm,
 * src and d_perm.  Sequences must not overlap in the rollout layout.
 * Device errors: BAD_LAYOUT (perm entry or offsets out of range, a sequence named twice by perm,
 * overlapping sequences),
 * ZERO_LENGTH_SEQ, OVERFLOW (a slot reaches beyond dst_capacity_tokens); a slot that fails a check
 * moves nothing.
 */
dc_status dc_scatter(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len, const int32_t* d_perm,
                     const dc_field* fields, int32_t n_fields, int64_t dst_capacity_tokens,
                     const int64_t* d_dst_tok_off, void* d_ws, size_t ws_bytes, int32_t* d_status, void* hip_stream);

const char* dc_strerror(dc_status code);

#ifdef __cplusplus
}
#endif
#endif /* DC_H */
