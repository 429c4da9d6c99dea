// Device code of the group-relative advantage stage, shared by the kernel of its own and by the
// launch that runs it beside the balance workgroup.
#pragma once
#include "dc_device.h"
#include "dc_internal.h"

namespace dc {

constexpr int ADV_UNROLL = 16;                          // 4-token chunks in flight per lane

struct AdvArgs {
    int32_t        n_seq, n_groups, ddof, per_token;
    double         eps;
    const int64_t* src_tok_off;
    const int32_t* seq_len;
    const float*   reward;
    const int32_t* group_off;
    float*         adv_seq;
    int32_t*       status;
    const uint8_t* mask[DC_MAX_SRC_SHARDS];
    float*         adv_tok[DC_MAX_SRC_SHARDS];
};

// Advantage of sequence i, evaluated by a whole wave (all lanes return the same value):
// float64 arithmetic in index order, one rounding to float32.  The group's rewards are
// fetched one per lane (64 at a time) and then consumed in order from registers, so the
// wave pays one memory round trip for them instead of one per reward.
__device__ __forceinline__ float seq_advantage(const AdvArgs& a, int i) {
    if (a.n_groups <= 0) return 0.0f;
    const int lane = threadIdx.x & (WAVE - 1);
    // group of i: try the position it has when all groups have the same size, else bisect
    int g = (int)(((int64_t)i * a.n_groups) / a.n_seq);
    int g0 = a.group_off[g], g1 = a.group_off[g + 1];
    if (i < g0 || i >= g1) {
        int lo = 0, hi = a.n_groups;                    // invariant: group_off[lo] <= i
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (a.group_off[mid] <= i) lo = mid; else hi = mid;
        }
        g0 = a.group_off[lo];
        g1 = a.group_off[lo + 1];
    }
    if (g0 < 0 || g1 > a.n_seq || i < g0 || i >= g1) return 0.0f;   // bad group table (flagged elsewhere)
    const int G = g1 - g0;
    const uint32_t r0 = __float_as_uint(a.reward[g0]);
    const double ri = (double)a.reward[i];

    bool same = true;
    double sum = 0.0;
    for (int base = g0; base < g1; base += WAVE) {
        const int n = min(WAVE, g1 - base);
        const float mine = lane < n ? a.reward[base + lane] : 0.0f;
        for (int q = 0; q < n; ++q) {
            const uint32_t bits = (uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(mine), q);
            same = same && bits == r0;
            sum += (double)__uint_as_float(bits);
        }
    }
    if (same || G - a.ddof <= 0) return 0.0f;
    const double mean = sum / (double)G;
    double ss = 0.0;
    for (int base = g0; base < g1; base += WAVE) {
        const int n = min(WAVE, g1 - base);
        const float mine = lane < n ? a.reward[base + lane] : 0.0f;
        for (int q = 0; q < n; ++q) {
            const double d = (double)__uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(mine), q)) - mean;
            ss += d * d;
        }
    }
    const double sd = sqrt(ss / (double)(G - a.ddof));
    return (float)((ri - mean) / (sd + a.eps));
}

__device__ __forceinline__ u32x4 select_by_mask(uint32_t mk, uint32_t av) {
    u32x4 o;
    o.x = (mk & 0x000000FFu) ? av : 0u;
    o.y = (mk & 0x0000FF00u) ? av : 0u;
    o.z = (mk & 0x00FF0000u) ? av : 0u;
    o.w = (mk & 0xFF000000u) ? av : 0u;
    return o;
}

// The work of wave number wv: sequence wv (its advantage, then its tokens), and one entry of the
// group table to check.  All 64 lanes of the wave must call it.
__device__ __forceinline__ void advantage_wave(const AdvArgs& a, const SourceDesc& sd, int64_t wv) {
    const int N = a.n_seq;
    const int lane = threadIdx.x & (WAVE - 1);

    if (wv <= a.n_groups && lane == 0) {                 // group table: [0] = 0, non-decreasing, last = N
        const int g = (int)wv;
        const int32_t v = a.group_off[g];
        bool bad = v < 0 || v > N || (g == 0 && v != 0) || (g == a.n_groups && v != N);
        if (g < a.n_groups && a.group_off[g + 1] < v) bad = true;
        if (bad) set_status(a.status, DC_ERR_BAD_LAYOUT);
    }
    if (wv >= N) return;
    const int i = (int)wv;
    const float adv = seq_advantage(a, i);
    if (lane == 0) a.adv_seq[i] = adv;

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
    if (!a.per_token) return;

    const uint8_t* __restrict__ mask = a.mask[s];
    float* __restrict__ out = a.adv_tok[s];
    const uint32_t av = __float_as_uint(adv);
    const int64_t end = so + ln;
    const int64_t a4 = min(end, (so + 3) & ~int64_t(3));         // first 4-aligned token
    const int64_t e4 = max(a4, end & ~int64_t(3));               // end of the 4-aligned body
    // ragged head and tail: at most 3 tokens each
    if (lane < 3 && so + lane < a4) out[so + lane] = mask[so + lane] ? adv : 0.0f;
    if (lane >= 32 && lane < 35 && e4 + (lane - 32) < end) out[e4 + lane - 32] = mask[e4 + lane - 32] ? adv : 0.0f;
    // body: 4 tokens per lane and step, ADV_UNROLL steps in flight
    const int64_t c_end = e4 >> 2;
    for (int64_t c = (a4 >> 2) + lane; c < c_end; c += WAVE * ADV_UNROLL) {
        uint32_t mk[ADV_UNROLL];
#pragma unroll
        for (int u = 0; u < ADV_UNROLL; ++u) {
            const int64_t cu = c + u * WAVE;
            mk[u] = cu < c_end ? load4(mask + cu * 4) : 0u;
        }
#pragma unroll
        for (int u = 0; u < ADV_UNROLL; ++u) {
            const int64_t cu = c + u * WAVE;
            if (cu < c_end) store16(out + cu * 4, select_by_mask(mk[u], av));
        }
    }
}

// What the host side fills in for either launch.
AdvArgs make_adv_args(int32_t n_seq, const SourceDesc& src, const int64_t* d_src_tok_off, const int32_t* d_seq_len,
                      const float* d_reward, const int32_t* d_group_off, int32_t n_groups, double eps, int32_t ddof,
                      const uint8_t* const* mask_base, float* d_adv_seq, float* const* adv_tok_base, int32_t* d_status);
// waves the stage needs: one per sequence, and one per entry of the group table
inline int64_t adv_waves(int32_t n_seq, int32_t n_groups) { return n_seq > n_groups + 1 ? n_seq : n_groups + 1; }

}  // namespace dc
