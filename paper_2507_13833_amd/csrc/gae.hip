// Generalized advantage estimation (Schulman et al. 2016, arXiv 1506.02438, eqs. 11-16) over the
// loss-bearing tokens of every sequence, in the rollout layout: the advantage stage of PPO
// (Sec. 7.1 evaluates PPO with a critic; App. B Table 2 "advantage"), the counterpart of the
// group-relative advantage.  Outputs per token: the advantage and the value target.
//
// With t_1 < ... < t_m the loss-bearing tokens of a sequence:
//   delta_k = r_k + gamma V[t_{k+1}] - V[t_k]   (V[t_{m+1}] = 0; r_k = KL penalty, plus the score on t_m)
//   A_k     = delta_k + gamma lambda A_{k+1},   ret_k = A_k + V[t_k]
// a first-order linear recurrence running backwards in time.  A workgroup of GAE_WAVES
// wavefronts shares one sequence and walks it from the end; per iteration a wave takes 512
// tokens, a lane 8 consecutive ones (two aligned 16-byte groups of the value array), lane 0 of
// wave 0 the latest.  Inside an iteration
//   * "gamma V of the next loss-bearing token" is a copy from the nearest earlier lane (or wave)
//     that holds one, not arithmetic;
//   * each lane folds its tokens into one affine map A_after = P A_in + B, the lanes' maps are
//     composed by a 6-step DPP scan, the waves' maps through LDS, and each lane then replays its
//     tokens from the state entering it;
//   * a wave whose 512 tokens all bear loss (the inside of a response) never looks at a mask
//     again; a wave without any loss-bearing token (a prompt) only writes zeros;
//   * the outputs leave through a transpose in LDS, so that a store instruction writes 64
//     consecutive 16-byte chunks (a lane's own 8 tokens are 32 bytes: two instructions that
//     each write every other 16 bytes, which streaming stores handle at a third of the rate).
// All arithmetic is float64 (the kernel is bound by HBM, not by the vector unit: 13 B per token,
// 21 with the KL penalty); outputs are rounded once to float32.
// Measured rationale: one wave per sequence left the longest sequence (36 K tokens, 141 dependent
// blocks) running alone for 160 us; with two waves it is still 36 dependent iterations, which
// run on alone when the sequence's workgroup starts late, so the first workgroups of the grid
// look for long sequences and start those; anything derived from a loaded mask word at load time makes
// the wave wait for the loads it has just issued (the prefetch ring keeps the raw words);
// plain loads with streaming stores beat both all-plain and all-streaming accesses (every line
// of the value array is touched by two load instructions, 32 bytes apart per lane).
#include <algorithm>
#include "dc_device.h"
#include "dc_internal.h"
#include "dc_lanes.h"

namespace dc {

constexpr int GAE_WAVES = 2;                 // waves that share one sequence

struct GaeArgs {
    int32_t        n_seq, use_kl;
    double         gamma, decay, kl_coef;            // decay = gamma * lambda
    int32_t        n_early, long_len;                // workgroups that start long sequences early; what counts as long
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

constexpr int GAE_TPL = 8;                   // tokens per lane: two aligned 16-byte groups of the value array

// One lane's 8 consecutive tokens: elements x0 .. x0+7 of the shard's buffers (x0 a multiple of 8).
template <bool KL>
struct GaeLane {
    float    v[GAE_TPL];                       // values (0 outside the sequence)
    float    lp[KL ? GAE_TPL : 1], rf[KL ? GAE_TPL : 1];   // log-probabilities, policy and reference (KL penalty only)
    uint32_t m[2];                             // the 8 mask bytes as loaded (0 outside the sequence); nothing is
                                               // derived from them before the lane's turn comes: a use here would make
                                               // the wave wait for the loads it has only just issued
    uint32_t inside;                           // bit t: token t belongs to the sequence
};

__device__ __forceinline__ uint32_t nonzero_bytes(uint32_t m) {
    return ((m & 0x000000FFu) ? 1u : 0u) | ((m & 0x0000FF00u) ? 2u : 0u) |
           ((m & 0x00FF0000u) ? 4u : 0u) | ((m & 0xFF000000u) ? 8u : 0u);
}

template <bool KL>
__device__ __forceinline__ void load_lane(const float* __restrict__ V, const uint8_t* __restrict__ M,
                                          const float* __restrict__ LP, const float* __restrict__ RF,
                                          int64_t x0, bool live, int64_t so, int64_t end, GaeLane<KL>& g) {
    if (live && x0 >= so && x0 + GAE_TPL <= end) {        // all 8 tokens inside the sequence: vector loads
        const f32x4 va = *reinterpret_cast<const f32x4*>(V + x0), vb = *reinterpret_cast<const f32x4*>(V + x0 + 4);
        g.m[0] = *reinterpret_cast<const uint32_t*>(M + x0);
        g.m[1] = *reinterpret_cast<const uint32_t*>(M + x0 + 4);
        g.v[0] = va.x; g.v[1] = va.y; g.v[2] = va.z; g.v[3] = va.w;
        g.v[4] = vb.x; g.v[5] = vb.y; g.v[6] = vb.z; g.v[7] = vb.w;
        g.inside = 0xFFu;
        if constexpr (KL) {
            const f32x4 pa = *reinterpret_cast<const f32x4*>(LP + x0), pb = *reinterpret_cast<const f32x4*>(LP + x0 + 4);
            const f32x4 ra = *reinterpret_cast<const f32x4*>(RF + x0), rb = *reinterpret_cast<const f32x4*>(RF + x0 + 4);
            g.lp[0] = pa.x; g.lp[1] = pa.y; g.lp[2] = pa.z; g.lp[3] = pa.w;
            g.lp[4] = pb.x; g.lp[5] = pb.y; g.lp[6] = pb.z; g.lp[7] = pb.w;
            g.rf[0] = ra.x; g.rf[1] = ra.y; g.rf[2] = ra.z; g.rf[3] = ra.w;
            g.rf[4] = rb.x; g.rf[5] = rb.y; g.rf[6] = rb.z; g.rf[7] = rb.w;
        }
    } else {                                              // the sequence starts or ends inside, or lies elsewhere
        g.m[0] = 0; g.m[1] = 0; g.inside = 0;
#pragma unroll
        for (int t = 0; t < GAE_TPL; ++t) g.v[t] = 0.0f;
#pragma unroll
        for (int t = 0; t < (KL ? GAE_TPL : 1); ++t) { g.lp[t] = 0.0f; g.rf[t] = 0.0f; }
        if (live) {
#pragma unroll
            for (int t = 0; t < GAE_TPL; ++t) {
                const int64_t x = x0 + t;
                if (x >= so && x < end) {
                    g.inside |= 1u << t;
                    g.v[t] = V[x];
                    g.m[t >> 2] |= (uint32_t)M[x] << (8 * (t & 3));
                    if constexpr (KL) { g.lp[t] = LP[x]; g.rf[t] = RF[x]; }
                }
            }
        }
    }
}

// ---- cross-lane moves of doubles through DPP (two 32-bit moves; nothing touches LDS) ----
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ double dpp_mov_f64(double old, double v) {
    const uint64_t o = (uint64_t)__double_as_longlong(old), x = (uint64_t)__double_as_longlong(v);
    const uint32_t lo = dpp_mov<CTRL, ROW_MASK>((uint32_t)o, (uint32_t)x);
    const uint32_t hi = dpp_mov<CTRL, ROW_MASK>((uint32_t)(o >> 32), (uint32_t)(x >> 32));
    return __longlong_as_double((long long)((uint64_t)lo | ((uint64_t)hi << 32)));
}
// One step of the inclusive scan of affine maps x -> P x + B in lane order: my map is applied
// after the map arriving from the lower lane; lanes that receive nothing see the identity.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ void affine_scan_step(double& P, double& B) {
    const double Pp = dpp_mov_f64<CTRL, ROW_MASK>(1.0, P), Bp = dpp_mov_f64<CTRL, ROW_MASK>(0.0, B);
    B = P * Bp + B;
    P = P * Pp;
}
__device__ __forceinline__ double readlane_f64(double v, int src) {
    const uint64_t x = (uint64_t)__double_as_longlong(v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, src);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), src);
    return __longlong_as_double((long long)((uint64_t)lo | ((uint64_t)hi << 32)));
}

constexpr int GAE_SET = 32;                  // sequences among which one may be started early
__device__ __forceinline__ bool gae_is_long(int32_t ln, int32_t long_len) { return ln >= long_len && ln <= DC_MAX_SEQ_LEN; }
// The longest long sequence among set, set + n_early, set + 2 n_early, ... (GAE_SET of them; ties: the lowest
// index), or -1; every wave that asks gets the same answer.
__device__ __forceinline__ int gae_longest_of_set(const GaeArgs& a, int set, int lane) {
    const int k = lane & (GAE_SET - 1);
    const int64_t idx = (int64_t)set + (int64_t)k * a.n_early;
    int32_t ln = 0;
    if (idx < a.n_seq) ln = a.seq_len[idx];
    long long key = gae_is_long(ln, a.long_len) ? (((long long)ln << 8) | (long long)(GAE_SET - 1 - k)) : -1ll;
#pragma unroll
    for (int d = GAE_SET / 2; d >= 1; d >>= 1) {
        const long long o = __shfl_xor(key, d, WAVE);
        key = o > key ? o : key;
    }
    return key < 0 ? -1 : set + (GAE_SET - 1 - (int)(key & 0xFF)) * a.n_early;
}

// Iterations whose loads are in flight ahead of the one worked on.
template <bool KL> constexpr int GAE_AHEAD = 2;

// One workgroup of NW waves per sequence.  An iteration covers NW * 512 tokens, wave 0 the
// latest 512 of them, lane 0 of a wave its latest 8.  The waves exchange two things through LDS:
// gamma * V of each wave's earliest loss-bearing token (a later wave's first loss-bearing token
// needs it), and each wave's composed map, from which every wave derives the state entering its
// tokens and the state carried to the next iteration.  Two barriers per iteration; every wave
// of the workgroup runs the same number of iterations (a wave whose lanes all lie before the
// sequence's start just takes part in the barriers).
template <int NW, bool KL>
__global__ __launch_bounds__(NW * WAVE) void gae_kernel(GaeArgs a, SourceDesc sd) {
    constexpr int AHEAD = GAE_AHEAD<KL>;
    constexpr int T = GAE_TPL;
    __shared__ double s_u[NW], s_P[NW], s_B[NW];
    __shared__ int32_t s_has[NW];
    __shared__ __attribute__((aligned(16))) float s_stage[NW][2 * WAVE * GAE_TPL];   // a wave's outputs on their way out
    const int lane = threadIdx.x & (WAVE - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / WAVE));
    // One workgroup per sequence, in index order, behind n_early workgroups that each start the longest
    // sequence of a set of GAE_SET (every n_early-th sequence from their own index on) if it is a long one:
    // a 36 K-token sequence is 36 dependent iterations, and started late it runs on alone after the rest.
    int i = (int)blockIdx.x - a.n_early;
    const bool early = i < 0;
    if (early || gae_is_long(a.seq_len[i], a.long_len)) {          // uniform over the workgroup
        const int set = early ? (int)blockIdx.x : i % a.n_early;
        const int longest = gae_longest_of_set(a, set, lane);
        if (early ? longest < 0 : longest == i) return;            // nothing to start early / started early
        if (early) i = __builtin_amdgcn_readfirstlane(longest);
    }
    int s = 0;
    while (s + 1 < sd.n_src && i >= sd.seq_off[s + 1]) ++s;
    const int64_t so = a.src_tok_off[i];
    const int32_t ln = a.seq_len[i];
    if (ln <= 0 || ln > DC_MAX_SEQ_LEN) {                          // uniform over the workgroup
        if (threadIdx.x == 0) set_status(a.status, DC_ERR_ZERO_LENGTH_SEQ);
        return;
    }
    if (so < 0 || so + ln > sd.tokens[s] || (i + 1 < sd.seq_off[s + 1] && a.src_tok_off[i + 1] < so + ln)) {
        if (threadIdx.x == 0) set_status(a.status, DC_ERR_BAD_LAYOUT);   // outside its buffer or overlapping the next
        return;
    }
    const float* __restrict__ V = a.value[s];
    const uint8_t* __restrict__ M = a.mask[s];
    const float* __restrict__ LP = a.logp[s];
    const float* __restrict__ RF = a.ref[s];
    float* __restrict__ ADV = a.adv[s];
    float* __restrict__ RET = a.ret[s];
    const int64_t end = so + ln;
    const int64_t q_lo = so >> 3, q_hi = (end - 1) >> 3;          // aligned 8-token lane groups the sequence touches
    const double gamma = a.gamma, decay = a.decay, klc = a.kl_coef;
    constexpr int STEP = NW * WAVE;                                // lane groups per iteration
    double decay_pow_T = 1.0;                                      // decay^8: a lane's multiplier when all its tokens bear loss
#pragma unroll
    for (int t = 0; t < T; ++t) decay_pow_T *= decay;

    // carried from iteration to iteration (uniform): A of the next loss-bearing token, and gamma * its
    // value, which starts out as the sequence's score (so the score lands on the last such token)
    double A_carry = 0.0, U_carry = (double)a.reward[i];

    GaeLane<KL> ring[AHEAD > 0 ? AHEAD : 1];
#pragma unroll
    for (int k = 0; k < AHEAD; ++k) {
        const int64_t q = q_hi - (int64_t)k * STEP - w * WAVE - lane;
        load_lane<KL>(V, M, LP, RF, q * T, q >= q_lo, so, end, ring[k]);
    }
    for (int64_t top = q_hi; top >= q_lo; top -= STEP) {
        const int64_t q = top - w * WAVE - lane;                   // my lane group; lane 0 of wave 0 holds the latest one
        GaeLane<KL> cur;
        if constexpr (AHEAD > 0) {
            cur = ring[0];
#pragma unroll
            for (int k = 0; k + 1 < AHEAD; ++k) ring[k] = ring[k + 1];
            const int64_t qn = q - (int64_t)AHEAD * STEP;
            load_lane<KL>(V, M, LP, RF, qn * T, qn >= q_lo, so, end, ring[AHEAD - 1]);
        } else {
            load_lane<KL>(V, M, LP, RF, q * T, q >= q_lo, so, end, cur);
        }
        const uint32_t loss = nonzero_bytes(cur.m[0]) | (nonzero_bytes(cur.m[1]) << 4);   // bit t: token t bears loss
        const uint64_t holders = __ballot(loss != 0);              // lanes of my wave with a loss-bearing token
        const bool any = holders != 0ull;                          // uniform over the wave
        // uniform: every lane that holds tokens of the sequence at all holds 8 loss-bearing ones (the
        // inside of a response); then no mask is looked at again
        const bool solid = any && __ballot(loss != 0xFFu && cur.inside != 0u) == 0ull;

        // ---- gamma * V of my earliest loss-bearing token; the wave's earliest goes to the other waves ----
        double U_last;
        if (solid) {
            U_last = gamma * (double)cur.v[0];
        } else {
            float first = cur.v[T - 1];
#pragma unroll
            for (int t = T - 2; t >= 0; --t)
                if (loss & (1u << t)) first = cur.v[t];
            U_last = gamma * (double)first;
        }
        const double U_wave = readlane_f64(U_last, any ? 63 - __builtin_clzll(holders) : 0);
        if (lane == 0) { s_has[w] = any ? 1 : 0; s_u[w] = U_wave; }
        __syncthreads();
        double U_w = U_carry, U_next = U_carry;                    // entering my wave / carried to the next iteration
#pragma unroll
        for (int k = 0; k < NW; ++k) {
            const bool h = s_has[k] != 0;
            const double u = s_u[k];
            if (h && k < w) U_w = u;
            if (h) U_next = u;
        }

        // ---- my tokens, latest first: r[t] = what token t adds to decay * A (its TD residual), and the lane's map
        // A_after = P * A_in + B; then the inclusive scan of the lanes' maps (rows of 16 lanes, then across rows) ----
        double r[T], Pi = 1.0, Bi = 0.0;
        if (solid) {
            double u = dpp_mov_f64<DPP_WAVE_SHR1>(U_w, U_last);    // gamma * V[0] of the lane before mine; lane 0: U_w
            double B = 0.0;
#pragma unroll
            for (int t = T - 1; t >= 0; --t) {
                const double vt = (double)cur.v[t];
                r[t] = u - vt;
                if constexpr (KL) r[t] = __builtin_fma(-klc, (double)cur.lp[t] - (double)cur.rf[t], r[t]);
                B = __builtin_fma(decay, B, r[t]);
                u = gamma * vt;
            }
            Pi = decay_pow_T; Bi = B;
        } else if (any) {
            const uint64_t before = holders & ((1ull << lane) - 1ull);        // lanes with later tokens than mine
            const int from = before ? 63 - __builtin_clzll(before) : 0;
            const double U_from = __shfl(U_last, from, WAVE);
            double u = before ? U_from : U_w, P = 1.0, B = 0.0;
#pragma unroll
            for (int t = T - 1; t >= 0; --t) {
                const double vt = (double)cur.v[t];
                r[t] = u - vt;
                if constexpr (KL) r[t] = __builtin_fma(-klc, (double)cur.lp[t] - (double)cur.rf[t], r[t]);
                if (loss & (1u << t)) {
                    B = __builtin_fma(decay, B, r[t]);
                    P = decay * P;
                    u = gamma * vt;
                }
            }
            Pi = P; Bi = B;
        }
        if (any) {
            affine_scan_step<DPP_ROW_SHR1>(Pi, Bi);
            affine_scan_step<DPP_ROW_SHR2>(Pi, Bi);
            affine_scan_step<DPP_ROW_SHR4>(Pi, Bi);
            affine_scan_step<DPP_ROW_SHR8>(Pi, Bi);
            affine_scan_step<DPP_ROW_BCAST15, 0xA>(Pi, Bi);
            affine_scan_step<DPP_ROW_BCAST31, 0xC>(Pi, Bi);
        }
        if (lane == WAVE - 1) { s_P[w] = Pi; s_B[w] = Bi; }       // the wave's whole map (identity without loss)
        __syncthreads();
        double A_w = A_carry, A_next = A_carry;                    // entering my wave / carried to the next iteration
#pragma unroll
        for (int k = 0; k < NW; ++k) {
            const double Pk = s_P[k], Bk = s_B[k];
            if (k == w) A_w = A_next;
            A_next = __builtin_fma(Pk, A_next, Bk);
        }

        // ---- outputs: replay my tokens from the state entering my lane ----
        float oa[T], orr[T];
#pragma unroll
        for (int t = 0; t < T; ++t) { oa[t] = 0.0f; orr[t] = 0.0f; }
        if (any) {
            // the maps of all lanes before mine (identity for lane 0), applied to the state entering the wave
            const double Pe = dpp_mov_f64<DPP_WAVE_SHR1>(1.0, Pi), Be = dpp_mov_f64<DPP_WAVE_SHR1>(0.0, Bi);
            double A = __builtin_fma(Pe, A_w, Be);
            if (solid) {
#pragma unroll
                for (int t = T - 1; t >= 0; --t) {
                    A = __builtin_fma(decay, A, r[t]);
                    oa[t] = (float)A;
                    orr[t] = (float)(A + (double)cur.v[t]);
                }
            } else {
#pragma unroll
                for (int t = T - 1; t >= 0; --t)
                    if (loss & (1u << t)) {
                        A = __builtin_fma(decay, A, r[t]);
                        oa[t] = (float)A;
                        orr[t] = (float)(A + (double)cur.v[t]);
                    }
            }
        }
        // ---- stores, through a transpose in LDS: a lane's 8 tokens are 32 bytes, and 16 bytes per lane at a
        // 32-byte stride, the other halves in a second instruction, is a pattern that streaming stores write at
        // a third of the rate of 64 consecutive 16-byte chunks (2.3 against 6.3 TB/s, write-only probe).
        // Memory order runs against lane order; the wave's window starts at lane 63's first token.
        if (__ballot(cur.inside != 0u) != 0ull) {                  // uniform: some token of the window lies inside
            float* st_a = s_stage[w];
            float* st_r = st_a + WAVE * T;
            const int mine = (WAVE - 1 - lane) * T;
            f32x4 o;
            o.x = oa[0]; o.y = oa[1]; o.z = oa[2]; o.w = oa[3];
            *reinterpret_cast<f32x4*>(st_a + mine) = o;
            o.x = oa[4]; o.y = oa[5]; o.z = oa[6]; o.w = oa[7];
            *reinterpret_cast<f32x4*>(st_a + mine + 4) = o;
            o.x = orr[0]; o.y = orr[1]; o.z = orr[2]; o.w = orr[3];
            *reinterpret_cast<f32x4*>(st_r + mine) = o;
            o.x = orr[4]; o.y = orr[5]; o.z = orr[6]; o.w = orr[7];
            *reinterpret_cast<f32x4*>(st_r + mine + 4) = o;
            const int64_t base = (top - (int64_t)w * WAVE - (WAVE - 1)) * T;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int c = (u * WAVE + lane) * 4;               // my chunk of 4 tokens in this instruction
                const int64_t t0 = base + c;
                const f32x4 va = *reinterpret_cast<const f32x4*>(st_a + c);
                const f32x4 vr = *reinterpret_cast<const f32x4*>(st_r + c);
                if (t0 >= so && t0 + 4 <= end) {
                    __builtin_nontemporal_store(va, reinterpret_cast<f32x4*>(ADV + t0));
                    __builtin_nontemporal_store(vr, reinterpret_cast<f32x4*>(RET + t0));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (t0 + e >= so && t0 + e < end) { ADV[t0 + e] = va[e]; RET[t0 + e] = vr[e]; }
                }
            }
        }
        A_carry = A_next;
        U_carry = U_next;
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
    // long: at least twice the mean (the buffers' sizes bound the lengths' sum) and at least 4 iterations
    int64_t tokens = 0;
    for (int s = 0; s < src.n_src; ++s) tokens += src.tokens[s];
    const int64_t twice_mean = 2 * (tokens / n_seq);
    a.long_len = (int32_t)std::min<int64_t>(std::max<int64_t>(twice_mean, 4 * GAE_WAVES * WAVE * GAE_TPL), INT32_MAX);
    a.n_early = (n_seq + GAE_SET - 1) / GAE_SET;
    const unsigned grid = (unsigned)(n_seq + a.n_early);
    for (int s = 0; s < DC_MAX_SRC_SHARDS; ++s) {
        const bool on = s < src.n_src;
        a.value[s] = on ? value_base[s] : nullptr;
        a.mask[s] = on ? mask_base[s] : nullptr;
        a.logp[s] = on && a.use_kl ? logp_base[s] : nullptr;
        a.ref[s] = on && a.use_kl ? ref_base[s] : nullptr;
        a.adv[s] = on ? adv_base[s] : nullptr;
        a.ret[s] = on ? ret_base[s] : nullptr;
    }
    if (a.use_kl)
        hipLaunchKernelGGL((gae_kernel<GAE_WAVES, true>), dim3(grid), dim3(GAE_WAVES * WAVE), 0, st, a, src);
    else
        hipLaunchKernelGGL((gae_kernel<GAE_WAVES, false>), dim3(grid), dim3(GAE_WAVES * WAVE), 0, st, a, src);
    return hipGetLastError();
}

}  // namespace dc
