/*
 * CPU oracle for the Data Coordinator reshard path.  TEST INFRASTRUCTURE ONLY:
 * the product (the HIP library) never links, loads or calls anything here.
 *
 * Plain, slow, single-threaded C written from the paper's statement of each
 * step.  No blocking, fusion or reordering beyond what the algorithm states.
 * All pointers are host pointers; the caller owns every buffer.
 *
 *   dco_balance          Algorithm 1 "Constrained LPT Load Balancing" (Sec. 6,
 *                        "Load Balancing"): longest sequence first, each to the
 *                        least-loaded worker that is not full.
 *   dco_group_advantage  group-relative (GRPO, Sec. 2 / Sec. 1 payload list)
 *                        advantage of each response: reward minus its prompt
 *                        group's mean over the group's std; float64, rounded
 *                        once to float32.  The paper names the stage
 *                        (App. B, Table 2 "advantage") but prints no formula;
 *                        the readings taken are listed at each function.
 *   dco_adv_broadcast    per-token advantage in the rollout layout.
 *   dco_gae              the PPO counterpart of the two above (Sec. 7.1 evaluates
 *                        PPO with a critic; the paper prints no formula):
 *                        generalized advantage estimation, Schulman et al. 2016
 *                        (arXiv 1506.02438) eqs. 11-16, over the loss-bearing
 *                        tokens of each sequence; float64, rounded once.
 *   dco_plan             packed training layout: shard token offsets,
 *                        next-fit micro-batches under a token budget,
 *                        per-micro-batch cu_seqlens.  (Sec. 6 "Distributed
 *                        Databuffer": redistribution between stages whose DP
 *                        sizes differ; the packing itself is a reading of
 *                        that passage, the paper's own batches are padded.)
 *   dco_gather           per-sequence copy rollout layout -> training layout.
 *   dco_scatter          the same copy backwards (training layout -> rollout
 *                        layout), for fields a training-layout stage produced
 *                        (App. B, Table 2: the collect / concat side of a stage
 *                        transition).
 *
 * Return value: 0 on success, a small positive code on invalid input.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

enum { DCO_OK = 0, DCO_BAD_ARG = 1, DCO_NOT_DIVISIBLE = 2, DCO_SEQ_EXCEEDS_BUDGET = 3,
       DCO_ZERO_LENGTH = 4, DCO_NOMEM = 5 };

/* ------------------------------------------------------------------ */
/* Algorithm 1                                                          */
/* ------------------------------------------------------------------ */

/* The order in which Algorithm 1 hands the sequences out: longest first, sequences of equal
 * length in ascending index order (the reading taken where the paper leaves ties open). */
static const int32_t* g_len_of;
static int longer_first(const void* pa, const void* pb) {
    const int32_t a = *(const int32_t*)pa, b = *(const int32_t*)pb;
    if (g_len_of[a] != g_len_of[b]) return g_len_of[a] > g_len_of[b] ? -1 : 1;
    return a < b ? -1 : (a > b);
}

/*
 * Algorithm 1, written from what it computes: the sequences are taken longest first, and each
 * goes to the worker whose (load, id) pair is lexicographically smallest among the workers that
 * still hold fewer than C sequences; that worker's load grows by the sequence's length.  (The
 * paper finds that worker with a priority queue from which full workers are taken out and put
 * back; here it is found by looking at every worker.)
 * S[N] lengths, K workers.  cap = 0 takes the paper's C = N/K, for which N mod K must be 0;
 * cap > 0 replaces C (cap = N makes the cardinality test vacuous: textbook LPT).
 * Outputs: perm[N] = members of P_0, then P_1, ... each in the order they were added;
 * shard_seq_off[K+1] = CSR offsets of the P_k inside perm; shard_of_seq[N]; shard_load[K].
 */
int dco_balance(const int32_t* S, int32_t N, int32_t K, int32_t cap,
                int32_t* perm, int32_t* shard_seq_off, int32_t* shard_of_seq, int64_t* shard_load) {
    if (N < 0 || K < 1) return DCO_BAD_ARG;
    int64_t C;
    if (cap == 0) {
        if (N % K != 0) return DCO_NOT_DIVISIBLE;
        C = N / K;
    } else {
        if (cap < 0 || (int64_t)cap * K < N) return DCO_BAD_ARG;
        C = cap;
    }
    for (int32_t i = 0; i < N; ++i) if (S[i] <= 0) return DCO_ZERO_LENGTH;

    const size_t n1 = (size_t)(N > 0 ? N : 1);
    int32_t* order = (int32_t*)malloc(sizeof(int32_t) * n1);
    int32_t* taken_by = (int32_t*)malloc(sizeof(int32_t) * n1);     /* worker of the t-th sequence handed out */
    int32_t* held = (int32_t*)calloc((size_t)K, sizeof(int32_t));   /* |P_k| */
    if (!order || !taken_by || !held) { free(order); free(taken_by); free(held); return DCO_NOMEM; }

    for (int32_t i = 0; i < N; ++i) order[i] = i;
    g_len_of = S;
    qsort(order, (size_t)N, sizeof(int32_t), longer_first);

    for (int32_t k = 0; k < K; ++k) shard_load[k] = 0;
    for (int32_t t = 0; t < N; ++t) {
        int32_t to = -1;
        for (int32_t k = 0; k < K; ++k) {
            if (held[k] >= C) continue;                              /* full: not a candidate */
            if (to < 0 || shard_load[k] < shard_load[to]) to = k;    /* equal loads: the smaller id stays */
        }
        taken_by[t] = to;
        held[to] += 1;
        shard_load[to] += S[order[t]];
    }

    /* lay the P_k out one after the other, members in the order they were added */
    shard_seq_off[0] = 0;
    for (int32_t k = 0; k < K; ++k) shard_seq_off[k + 1] = shard_seq_off[k] + held[k];
    memset(held, 0, sizeof(int32_t) * (size_t)K);
    for (int32_t t = 0; t < N; ++t) {
        const int32_t k = taken_by[t], u = order[t];
        perm[shard_seq_off[k] + held[k]++] = u;
        shard_of_seq[u] = k;
    }
    free(order); free(taken_by); free(held);
    return DCO_OK;
}

/* ------------------------------------------------------------------ */
/* Group-relative advantage                                             */
/* ------------------------------------------------------------------ */

/*
 * For each prompt group g = [group_off[g], group_off[g+1]) with rewards r_1..r_G:
 *   mean = (1/G) sum r,  var = sum (r-mean)^2 / (G - ddof),
 *   A_i  = (r_i - mean) / (sqrt(var) + eps)
 * in float64, rounded once to float32.  Readings where the paper is silent:
 * eps is added to the std outside the root; a group with G - ddof <= 0 gets 0;
 * a group whose rewards are all bit-identical gets exactly +0.
 */
int dco_group_advantage(const float* reward, const int32_t* group_off, int32_t n_groups,
                        double eps, int32_t ddof, float* adv_seq) {
    if (n_groups < 0 || ddof < 0) return DCO_BAD_ARG;
    for (int32_t g = 0; g < n_groups; ++g) {
        int32_t a = group_off[g], b = group_off[g + 1];
        if (b < a) return DCO_BAD_ARG;
        int32_t G = b - a;
        if (G == 0) continue;
        int all_same = 1;
        for (int32_t i = a + 1; i < b; ++i)
            if (memcmp(&reward[i], &reward[a], sizeof(float)) != 0) { all_same = 0; break; }
        if (all_same || G - ddof <= 0) {
            for (int32_t i = a; i < b; ++i) adv_seq[i] = 0.0f;
            continue;
        }
        double sum = 0.0;
        for (int32_t i = a; i < b; ++i) sum += (double)reward[i];
        double mean = sum / (double)G;
        double ss = 0.0;
        for (int32_t i = a; i < b; ++i) { double d = (double)reward[i] - mean; ss += d * d; }
        double sd = sqrt(ss / (double)(G - ddof));
        for (int32_t i = a; i < b; ++i)
            adv_seq[i] = (float)(((double)reward[i] - mean) / (sd + eps));
    }
    return DCO_OK;
}

/*
 * Per-token advantage inside ONE rollout shard holding sequences
 * [seq_begin, seq_end): token t of sequence i gets adv_seq[i] where mask != 0 and
 * +0.0 elsewhere (selection, not multiplication).  mask / adv_tok point at the
 * shard's packed buffers; src_tok_off[i] is sequence i's first element in them.
 */
int dco_adv_broadcast(const float* adv_seq, const int32_t* S, const int64_t* src_tok_off,
                      int32_t seq_begin, int32_t seq_end, const uint8_t* mask, float* adv_tok) {
    for (int32_t i = seq_begin; i < seq_end; ++i) {
        int64_t base = src_tok_off[i];
        for (int32_t t = 0; t < S[i]; ++t)
            adv_tok[base + t] = mask[base + t] ? adv_seq[i] : 0.0f;
    }
    return DCO_OK;
}

/*
 * Generalized advantage estimation inside ONE rollout shard holding sequences
 * [seq_begin, seq_end).  Let t_1 < ... < t_m be the loss-bearing tokens (mask != 0)
 * of sequence i; tokens without loss are transparent (the recursion steps over them).
 *   r_k     = -kl_coef * (logp[t_k] - ref_logp[t_k])     (per-token KL penalty, if kl_coef != 0)
 *             + reward[i] if k = m                       (the sequence's score sits on its last token)
 *   delta_k = r_k + gamma * V[t_{k+1}] - V[t_k],  V[t_{m+1}] = 0      (TD residual, eq. 11 / 16)
 *   A_k     = delta_k + gamma * lambda * A_{k+1}, A_{m+1} = 0         (= sum_l (gamma lambda)^l delta_{k+l}, eq. 16)
 *   ret_k   = A_k + V[t_k]                                            (value target)
 * adv_tok / ret_tok get A_k / ret_k at t_k and +0.0 at every other token of the
 * sequence.  All arithmetic in float64, each output rounded once to float32.
 * logp / ref_logp may be NULL when kl_coef == 0.
 */
int dco_gae(const float* reward, const int32_t* S, const int64_t* src_tok_off,
            int32_t seq_begin, int32_t seq_end, const float* value, const uint8_t* mask,
            const float* logp, const float* ref_logp, double gamma, double lambda, double kl_coef,
            float* adv_tok, float* ret_tok) {
    if (kl_coef != 0.0 && (!logp || !ref_logp)) return DCO_BAD_ARG;
    for (int32_t i = seq_begin; i < seq_end; ++i) {
        const int64_t base = src_tok_off[i];
        double next_A = 0.0, next_V = 0.0;
        int seen_last = 0;
        for (int32_t t = S[i] - 1; t >= 0; --t) {
            const int64_t x = base + t;
            if (!mask[x]) { adv_tok[x] = 0.0f; ret_tok[x] = 0.0f; continue; }
            double r = 0.0;
            if (kl_coef != 0.0) r = -kl_coef * ((double)logp[x] - (double)ref_logp[x]);
            if (!seen_last) { r += (double)reward[i]; seen_last = 1; }
            const double V = (double)value[x];
            const double delta = r + gamma * next_V - V;
            const double A = delta + gamma * lambda * next_A;
            adv_tok[x] = (float)A;
            ret_tok[x] = (float)(A + V);
            next_A = A;
            next_V = V;
        }
    }
    return DCO_OK;
}

/* ------------------------------------------------------------------ */
/* Plan of the packed training layout                                   */
/* ------------------------------------------------------------------ */

/*
 * Output slots follow perm (shard after shard).  Shard p starts at
 * shard_tok_off[p]; shard_tok_off[p+1] = round_up(shard_tok_off[p] + load_p, align).
 * dst_tok_off[j] = first token of slot j; dst_tok_off[N] = shard_tok_off[K].
 * Micro-batches: next-fit in slot order inside a shard - a slot joins the open
 * micro-batch iff its tokens still fit under the budget, else it opens a new
 * one; a shard's first slot always opens one.  cu_seqlens: for micro-batch m
 * (slots [mb_seq_off[m], mb_seq_off[m+1])) a slice of n_m + 1 int32 starting at
 * index mb_seq_off[m] + m: 0, then running token totals.
 */
int dco_plan(const int32_t* S, int32_t N, const int32_t* perm, const int32_t* shard_seq_off, int32_t K,
             int64_t budget, int32_t align,
             int64_t* dst_tok_off, int64_t* shard_tok_off, int32_t* shard_mb_off,
             int32_t* mb_seq_off, int32_t* cu_seqlens, int32_t* n_mb) {
    if (N < 0 || K < 1 || align < 1 || budget < 1) return DCO_BAD_ARG;
    int32_t M = 0;
    int64_t pos = 0;
    shard_tok_off[0] = 0;
    for (int32_t p = 0; p < K; ++p) {
        shard_mb_off[p] = M;
        int64_t in_mb = 0;
        int32_t cu_at = 0;
        for (int32_t j = shard_seq_off[p]; j < shard_seq_off[p + 1]; ++j) {
            int64_t len = S[perm[j]];
            if (len <= 0) return DCO_ZERO_LENGTH;
            if (len > budget) return DCO_SEQ_EXCEEDS_BUDGET;
            dst_tok_off[j] = pos;
            if (j == shard_seq_off[p] || in_mb + len > budget) {   /* open a micro-batch */
                mb_seq_off[M] = j;
                cu_at = j + M;
                cu_seqlens[cu_at] = 0;
                in_mb = 0;
                M += 1;
            }
            in_mb += len;
            cu_at += 1;
            cu_seqlens[cu_at] = (int32_t)in_mb;
            pos += len;
        }
        pos = (pos + align - 1) / align * align;
        shard_tok_off[p + 1] = pos;
    }
    shard_mb_off[K] = M;
    mb_seq_off[M] = N;
    dst_tok_off[N] = pos;
    *n_mb = M;
    return DCO_OK;
}

/* ------------------------------------------------------------------ */
/* Gather                                                               */
/* ------------------------------------------------------------------ */

/*
 * One field.  Sequence i lives in rollout shard s with
 * src_shard_seq_off[s] <= i < src_shard_seq_off[s+1], at element src_tok_off[i] of
 * src_base[s].  Slot j (sequence perm[j]) is copied, byte for byte, to element
 * dst_tok_off[j] of dst.
 */
int dco_gather(const int32_t* S, int32_t N, const int32_t* perm, const int64_t* src_tok_off,
               const int32_t* src_shard_seq_off, int32_t n_src, const void* const* src_base,
               void* dst, int32_t elem_bytes, const int64_t* dst_tok_off) {
    if (elem_bytes < 1) return DCO_BAD_ARG;
    for (int32_t j = 0; j < N; ++j) {
        int32_t i = perm[j];
        int32_t s = 0;
        while (s < n_src && !(src_shard_seq_off[s] <= i && i < src_shard_seq_off[s + 1])) ++s;
        if (s == n_src) return DCO_BAD_ARG;
        const char* from = (const char*)src_base[s] + src_tok_off[i] * elem_bytes;
        char* to = (char*)dst + dst_tok_off[j] * elem_bytes;
        memcpy(to, from, (size_t)S[i] * (size_t)elem_bytes);
    }
    return DCO_OK;
}

/*
 * Reverse of dco_gather for one field: slot j (sequence perm[j]) is copied, byte for
 * byte, from element dst_tok_off[j] of the training arena to the sequence's place in
 * its rollout buffer.  Elements of the rollout buffers that belong to no sequence
 * (padding between rows) are not touched.
 */
int dco_scatter(const int32_t* S, int32_t N, const int32_t* perm, const int64_t* src_tok_off,
                const int32_t* src_shard_seq_off, int32_t n_src, void* const* rollout_base,
                const void* arena, int32_t elem_bytes, const int64_t* dst_tok_off) {
    if (elem_bytes < 1) return DCO_BAD_ARG;
    for (int32_t j = 0; j < N; ++j) {
        int32_t i = perm[j];
        int32_t s = 0;
        while (s < n_src && !(src_shard_seq_off[s] <= i && i < src_shard_seq_off[s + 1])) ++s;
        if (s == n_src) return DCO_BAD_ARG;
        char* to = (char*)rollout_base[s] + src_tok_off[i] * elem_bytes;
        const char* from = (const char*)arena + dst_tok_off[j] * elem_bytes;
        memcpy(to, from, (size_t)S[i] * (size_t)elem_bytes);
    }
    return DCO_OK;
}
