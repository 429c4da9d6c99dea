// Generalized advantage estimation (Schulman et al. 2016, arXiv 1506.02438, eqs. 11-16) over the
// loss-bearing tokens of every sequence, in the rollout layout: the advantage stage of PPO
// (Sec. 7.1 evaluates PPO with a critic; App. B Table 2 "advantage"), the counterpart of the
// group-relative advantage.  Outputs per token: the advantage and the value target.
//
// With t_1 < ... < t_m the loss-bearing tokens of a sequence:
//   delta_k = r_k + gamma V[t_{k+1}] - V[t_k]   (V[t_{m+1}] = 0; r_k = KL penalty, plus the score on t_m)
//   A_k     = delta_k + gamma lambda A_{k+1},   ret_k = A_k + V[t_k]
// a first-order linear recurrence running backwards in time.  One wavefront per sequence walks
// it from the end in blocks of 256 tokens: lane l holds 4 consecutive tokens (one aligned
// 16-byte group of the value array), lane 0 the latest.  Inside a block
//   * "gamma V of the next loss-bearing token" is a copy from the nearest earlier lane that
//     holds one (ballot + one cross-lane read), not arithmetic;
//   * each lane folds its 4 tokens into one affine map A_out = P A_in + B, the maps are
//     composed by a 6-step wave scan, and each lane then replays its tokens from its A_in.
// All arithmetic is float64 (the vector unit runs it at half the float32 rate and the kernel
// is HBM-bound: 13 B per token, 21 with the KL penalty); outputs are rounded once to float32.
// The next block's loads are issued before the current block is worked on.
#include "dc_device.h"
#include "dc_internal.h"

namespace dc {

constexpr int GAE_BLOCK = 256;
constexpr int GAE_WAVES = GAE_BLOCK / WAVE;

struct GaeArgs {
    int32_t        n_seq, use_kl;
    double         gamma, decay, kl_coef;            // decay = gamma * lambda
    const int64_t* src_tok_off;
    const int32_t* seq_len;
    const float*   reward;
    int32_t*       status;
    const float*   value[DC_MAX_SRC_SHARDS];
    const uint8_t* mask[DC_MAX_SRC_SHARDS];
    const float*   logp[DC_MAX_SRC_SHARDS];
    const float*   ref[DC_MAX_SRC_SHARDS];
    float*         adv[DC_MAX_SRC_SHARDS];
    float*         ret[DC_MAX_SRC_SHARDS];
};

typedef float f32x4 __attribute__((ext_vector_type(4)));

// One lane's group of 4 tokens: elements x0 .. x0+3 of the shard's buffers.
struct GaeGroup {
    float    v[4];            // values (0 outside the sequence)
    float    lp[4], rf[4];    // log-probabilities under the policy and the reference (only with the KL penalty)
    uint32_t loss;            // bit e: token e belongs to the sequence and bears loss
    uint32_t inside;          // bit e: token e belongs to the sequence
};

__device__ __forceinline__ void load_group(const GaeArgs& a, const float* __restrict__ V, const uint8_t* __restrict__ M,
                                           const float* __restrict__ LP, const float* __restrict__ RF,
                                           int64_t x0, bool live, int64_t so, int64_t end, GaeGroup& g) {
    g.loss = 0; g.inside = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) { g.v[e] = 0.0f; g.lp[e] = 0.0f; g.rf[e] = 0.0f; }
    if (!live) return;
    if (x0 >= so && x0 + 4 <= end) {                      // whole group inside the sequence: vector loads
        const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(V + x0));
        const uint32_t m = load4(M + x0);
        g.v[0] = v.x; g.v[1] = v.y; g.v[2] = v.z; g.v[3] = v.w;
        g.inside = 0xFu;
        g.loss = ((m & 0x000000FFu) ? 1u : 0u) | ((m & 0x0000FF00u) ? 2u : 0u) |
                 ((m & 0x00FF0000u) ? 4u : 0u) | ((m & 0xFF000000u) ? 8u : 0u);
        if (a.use_kl) {
            const f32x4 p = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(LP + x0));
            const f32x4 r = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(RF + x0));
            g.lp[0] = p.x; g.lp[1] = p.y; g.lp[2] = p.z; g.lp[3] = p.w;
            g.rf[0] = r.x; g.rf[1] = r.y; g.rf[2] = r.z; g.rf[3] = r.w;
        }
    } else {                                              // first or last group of the sequence: per element
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t x = x0 + e;
            if (x >= so && x < end) {
                g.inside |= 1u << e;
                g.v[e] = V[x];
                if (M[x]) g.loss |= 1u << e;
                if (a.use_kl) { g.lp[e] = LP[x]; g.rf[e] = RF[x]; }
            }
        }
    }
}

__global__ __launch_bounds__(GAE_BLOCK) void gae_kernel(GaeArgs a, SourceDesc sd) {
    const int N = a.n_seq;
    const int lane = threadIdx.x & (WAVE - 1);
    const int64_t wv = (int64_t)blockIdx.x * GAE_WAVES + threadIdx.x / WAVE;    // one wave per sequence
    if (wv >= N) return;
    const int i = __builtin_amdgcn_readfirstlane((int)wv);
    int s = 0;
    while (s + 1 < sd.n_src && i >= sd.seq_off[s + 1]) ++s;
    const int64_t so = a.src_tok_off[i];
    const int32_t ln = a.seq_len[i];
    if (ln <= 0 || ln > DC_MAX_SEQ_LEN) {
        if (lane == 0) set_status(a.status, DC_ERR_ZERO_LENGTH_SEQ);
        return;
    }
    if (so < 0 || so + ln > sd.tokens[s] || (i + 1 < sd.seq_off[s + 1] && a.src_tok_off[i + 1] < so + ln)) {
        if (lane == 0) set_status(a.status, DC_ERR_BAD_LAYOUT);   // outside its buffer or overlapping the next
        return;
    }
    const float* __restrict__ V = a.value[s];
    const uint8_t* __restrict__ M = a.mask[s];
    const float* __restrict__ LP = a.logp[s];
    const float* __restrict__ RF = a.ref[s];
    float* __restrict__ ADV = a.adv[s];
    float* __restrict__ RET = a.ret[s];
    const int64_t end = so + ln;
    const int64_t q_lo = so >> 2, q_hi = (end - 1) >> 2;          // aligned 4-token groups the sequence touches
    const double gamma = a.gamma, decay = a.decay, klc = a.kl_coef;

    // carried from block to block (uniform): A of the next loss-bearing token, and gamma * its
    // value, which starts out as the sequence's score (so the score lands on the last such token)
    double A_carry = 0.0, U_carry = (double)a.reward[i];

    GaeGroup cur;
    load_group(a, V, M, LP, RF, (q_hi - lane) * 4, q_hi - lane >= q_lo, so, end, cur);
    for (int64_t qb = q_hi; qb >= q_lo; qb -= WAVE) {
        const int64_t q = qb - lane;                              // my group; lane 0 holds the latest one
        GaeGroup nxt;
        load_group(a, V, M, LP, RF, (q - WAVE) * 4, q - WAVE >= q_lo, so, end, nxt);

        // ---- gamma * V of the next loss-bearing token behind each lane's tokens ----
        const bool has = cur.loss != 0;
        const int e_first = has ? __builtin_ctz(cur.loss) : 0;    // my earliest loss-bearing token
        double U_last = 0.0;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (e == e_first) U_last = gamma * (double)cur.v[e];
        const uint64_t holders = __ballot(has);
        const uint64_t before = holders & ((1ull << lane) - 1ull);            // lanes with later tokens than mine
        const int from = before ? 63 - __builtin_clzll(before) : 0;
        const double U_from = __shfl(U_last, from, WAVE);
        const double U_in = before ? U_from : U_carry;

        // ---- my 4 tokens as one affine map A_out = P * A_in + B (latest token first) ----
        double rk[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) rk[e] = a.use_kl ? -klc * ((double)cur.lp[e] - (double)cur.rf[e]) : 0.0;
        double P = 1.0, B = 0.0, u = U_in;
#pragma unroll
        for (int e = 3; e >= 0; --e)
            if (cur.loss & (1u << e)) {
                const double delta = (rk[e] + u) - (double)cur.v[e];
                B = delta + decay * B;
                P = decay * P;
                u = gamma * (double)cur.v[e];
            }
        // ---- inclusive scan of the maps in lane order (an earlier lane's map is applied first) ----
        double Pi = P, Bi = B;
#pragma unroll
        for (int d = 1; d < WAVE; d <<= 1) {
            const double Pp = __shfl_up(Pi, d, WAVE), Bp = __shfl_up(Bi, d, WAVE);
            if (lane >= d) { Bi = Pi * Bp + Bi; Pi = Pi * Pp; }
        }
        const double Pe = __shfl_up(Pi, 1, WAVE), Be = __shfl_up(Bi, 1, WAVE);    // maps of all lanes before mine
        double A = lane == 0 ? A_carry : Pe * A_carry + Be;

        // ---- replay my tokens from A, write the outputs ----
        float oa[4], orr[4];
        u = U_in;
#pragma unroll
        for (int e = 3; e >= 0; --e) {
            oa[e] = 0.0f; orr[e] = 0.0f;
            if (cur.loss & (1u << e)) {
                const double delta = (rk[e] + u) - (double)cur.v[e];
                A = delta + decay * A;
                oa[e] = (float)A;
                orr[e] = (float)(A + (double)cur.v[e]);
                u = gamma * (double)cur.v[e];
            }
        }
        const int64_t x0 = q * 4;
        if (cur.inside == 0xFu) {
            f32x4 o; o.x = oa[0]; o.y = oa[1]; o.z = oa[2]; o.w = oa[3];
            __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(ADV + x0));
            f32x4 r; r.x = orr[0]; r.y = orr[1]; r.z = orr[2]; r.w = orr[3];
            __builtin_nontemporal_store(r, reinterpret_cast<f32x4*>(RET + x0));
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (cur.inside & (1u << e)) { ADV[x0 + e] = oa[e]; RET[x0 + e] = orr[e]; }
        }

        // ---- carry to the next (earlier) block ----
        A_carry = __shfl(A, WAVE - 1, WAVE);
        if (holders) U_carry = __shfl(U_last, 63 - __builtin_clzll(holders), WAVE);
        cur = nxt;
    }
}

hipError_t launch_gae(int32_t n_seq, const SourceDesc& src, const int64_t* d_src_tok_off, const int32_t* d_seq_len,
                      const float* d_reward, const float* const* value_base, const uint8_t* const* mask_base,
                      const float* const* logp_base, const float* const* ref_base, double gamma, double lambda,
                      double kl_coef, float* const* adv_base, float* const* ret_base, int32_t* d_status,
                      hipStream_t st) {
    if (n_seq == 0) return hipSuccess;
    GaeArgs a;
    a.n_seq = n_seq; a.use_kl = kl_coef != 0.0 ? 1 : 0;
    a.gamma = gamma; a.decay = gamma * lambda; a.kl_coef = kl_coef;
    a.src_tok_off = d_src_tok_off; a.seq_len = d_seq_len; a.reward = d_reward; a.status = d_status;
    for (int s = 0; s < DC_MAX_SRC_SHARDS; ++s) {
        const bool on = s < src.n_src;
        a.value[s] = on ? value_base[s] : nullptr;
        a.mask[s] = on ? mask_base[s] : nullptr;
        a.logp[s] = on && a.use_kl ? logp_base[s] : nullptr;
        a.ref[s] = on && a.use_kl ? ref_base[s] : nullptr;
        a.adv[s] = on ? adv_base[s] : nullptr;
        a.ret[s] = on ? ret_base[s] : nullptr;
    }
    const int64_t grid = ((int64_t)n_seq + GAE_WAVES - 1) / GAE_WAVES;
    hipLaunchKernelGGL(gae_kernel, dim3((unsigned)grid), dim3(GAE_BLOCK), 0, st, a, src);
    return hipGetLastError();
}

}  // namespace dc
