/*
 * CPU oracle for the Data Coordinator reshard path.  TEST INFRASTRUCTURE ONLY:
 * the product (the HIP library) never links, loads or calls anything here.
 *
 * Plain, slow, single-threaded C written from the paper's statement of each
 * step.  No blocking, fusion or reordering beyond what the algorithm states.
 * All pointers are host pointers; the caller owns every buffer.
 *
 *   dco_balance          Algorithm 1 "Constrained LPT Load Balancing" (Sec. 6,
 *                        "Load Balancing"): descending argsort, a min-heap of
 *                        (load, k) tuples, full workers popped, set aside in B
 *                        and pushed back.
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

typedef struct { int64_t load; int32_t k; } heap_item;

/* tuples compare lexicographically: smaller load first, then smaller k */
static int item_less(heap_item a, heap_item b) {
    if (a.load != b.load) return a.load < b.load;
    return a.k < b.k;
}

static void heap_push(heap_item* h, int32_t* n, heap_item x) {
    int32_t i = (*n)++;
    h[i] = x;
    while (i > 0) {
        int32_t p = (i - 1) / 2;
        if (!item_less(h[i], h[p])) break;
        heap_item t = h[i]; h[i] = h[p]; h[p] = t;
        i = p;
    }
}

static heap_item heap_pop_min(heap_item* h, int32_t* n) {
    heap_item top = h[0];
    h[0] = h[--(*n)];
    int32_t i = 0;
    for (;;) {
        int32_t l = 2 * i + 1, r = l + 1, m = i;
        if (l < *n && item_less(h[l], h[m])) m = l;
        if (r < *n && item_less(h[r], h[m])) m = r;
        if (m == i) break;
        heap_item t = h[i]; h[i] = h[m]; h[m] = t;
        i = m;
    }
    return top;
}

static const int32_t* g_sort_keys;
/* descending length; equal lengths keep ascending original index (stable) */
static int cmp_desc_stable(const void* a, const void* b) {
    int32_t ia = *(const int32_t*)a, ib = *(const int32_t*)b;
    if (g_sort_keys[ia] != g_sort_keys[ib]) return g_sort_keys[ia] > g_sort_keys[ib] ? -1 : 1;
    return ia < ib ? -1 : (ia > ib);
}

/*
 * Algorithm 1.  S[N] lengths, K workers, cap = 0 takes the paper's C = N/K
 * (N mod K must be 0); cap > 0 replaces C (cap = N makes the cardinality test
 * vacuous and the algorithm is then textbook LPT).
 * Outputs: perm[N] = members of P_0, then P_1, ... each in insertion order;
 * shard_seq_off[K+1] = CSR offsets of the P_k inside perm; shard_of_seq[N];
 * shard_load[K].
 */
int dco_balance(const int32_t* S, int32_t N, int32_t K, int32_t cap,
                int32_t* perm, int32_t* shard_seq_off, int32_t* shard_of_seq, int64_t* shard_load) {
    if (N < 0 || K < 1) return DCO_BAD_ARG;
    int64_t C;
    if (cap == 0) {
        if (N % K != 0) return DCO_NOT_DIVISIBLE;       /* Assert N mod K = 0 */
        C = N / K;
    } else {
        if (cap < 0 || (int64_t)cap * K < N) return DCO_BAD_ARG;
        C = cap;
    }
    for (int32_t i = 0; i < N; ++i) if (S[i] <= 0) return DCO_ZERO_LENGTH;

    int32_t* I = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    heap_item* H = (heap_item*)malloc(sizeof(heap_item) * (size_t)K);
    heap_item* B = (heap_item*)malloc(sizeof(heap_item) * (size_t)K);
    int32_t* count = (int32_t*)calloc((size_t)K, sizeof(int32_t));
    int32_t* worker_of_step = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    if (!I || !H || !B || !count || !worker_of_step) { free(I); free(H); free(B); free(count); free(worker_of_step); return DCO_NOMEM; }

    for (int32_t i = 0; i < N; ++i) I[i] = i;           /* I <- argsort(S, descending) */
    g_sort_keys = S;
    qsort(I, (size_t)N, sizeof(int32_t), cmp_desc_stable);

    int32_t hn = 0;                                     /* H <- {(0,k)} */
    for (int32_t k = 0; k < K; ++k) { heap_item x = {0, k}; heap_push(H, &hn, x); }

    for (int32_t t = 0; t < N; ++t) {                   /* for each u in I */
        int32_t u = I[t];
        int32_t bn = 0;                                 /* B <- empty */
        for (;;) {
            heap_item top = heap_pop_min(H, &hn);
            if (count[top.k] < C) {                     /* |P_k| < C */
                worker_of_step[t] = top.k;              /* P_k <- P_k U {u} */
                count[top.k] += 1;
                heap_item x = {top.load + S[u], top.k};
                heap_push(H, &hn, x);
                break;
            }
            B[bn++] = top;
        }
        for (int32_t b = 0; b < bn; ++b) heap_push(H, &hn, B[b]);
    }

    /* lay the P_k out one after the other, members in insertion order */
    shard_seq_off[0] = 0;
    for (int32_t k = 0; k < K; ++k) { shard_seq_off[k + 1] = shard_seq_off[k] + count[k]; shard_load[k] = 0; }
    memset(count, 0, sizeof(int32_t) * (size_t)K);
    for (int32_t t = 0; t < N; ++t) {
        int32_t k = worker_of_step[t], u = I[t];
        perm[shard_seq_off[k] + count[k]++] = u;
        shard_of_seq[u] = k;
        shard_load[k] += S[u];
    }
    free(I); free(H); free(B); free(count); free(worker_of_step);
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
