// Group-relative advantage (the GRPO "advantage" stage, App. B Table 2; advantages
// are part of the payload the Data Coordinator moves, Sec. 1) fused with its
// broadcast over the rollout layout's tokens.
//
// One launch.  Lanes 0..N-1 of the grid first write adv_seq[i].  Then every
// workgroup owns one tile of ADV_TILE tokens of one rollout shard: it finds the
// sequences that overlap the tile (binary search over the shard's increasing
// offsets), recomputes their advantages from the group's rewards (G float64
// additions each - cheaper than a second launch) into LDS, and streams the tile:
// 4 mask bytes in, 16 bytes of float32 out per lane and step (5 B/token, HBM-bound).
#include "dc_device.h"
#include "dc_internal.h"

namespace dc {

constexpr int ADV_BLOCK = 256;
constexpr int ADV_NSEG = SEG_BATCH + 4;                 // a 4-token chunk can reach 3 segments ahead

struct AdvArgs {
    int32_t        n_seq, n_groups, ddof, n_src;
    double         eps;
    const int64_t* src_tok_off;
    const int32_t* seq_len;
    const float*   reward;
    const int32_t* group_off;
    float*         adv_seq;
    int32_t*       status;
    int32_t        tile_off[DC_MAX_SRC_SHARDS + 1];     // first workgroup of each rollout shard
    const uint8_t* mask[DC_MAX_SRC_SHARDS];
    float*         adv_tok[DC_MAX_SRC_SHARDS];
};

// Advantage of sequence i (float64 arithmetic, one rounding to float32).
__device__ float seq_advantage(const AdvArgs& a, int i) {
    if (a.n_groups <= 0) return 0.0f;
    // group of i: last g with group_off[g] <= i
    int lo = 0, hi = a.n_groups;                        // invariant: group_off[lo] <= i
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.group_off[mid] <= i) lo = mid; else hi = mid;
    }
    const int g0 = a.group_off[lo], g1 = a.group_off[lo + 1];
    if (g0 < 0 || g1 > a.n_seq || i < g0 || i >= g1) return 0.0f;   // bad group table (flagged elsewhere)
    const int G = g1 - g0;
    const float r0 = a.reward[g0];
    bool same = true;
    double sum = 0.0;
    for (int q = g0; q < g1; ++q) {
        const float r = a.reward[q];
        same = same && (__float_as_uint(r) == __float_as_uint(r0));
        sum += (double)r;
    }
    if (same || G - a.ddof <= 0) return 0.0f;
    const double mean = sum / (double)G;
    double ss = 0.0;
    for (int q = g0; q < g1; ++q) {
        const double d = (double)a.reward[q] - mean;
        ss += d * d;
    }
    const double sd = sqrt(ss / (double)(G - a.ddof));
    return (float)(((double)a.reward[i] - mean) / (sd + a.eps));
}

struct AdvLds {
    int64_t start[ADV_NSEG];
    int32_t len[ADV_NSEG];
    float   adv[ADV_NSEG];
};

__global__ __launch_bounds__(ADV_BLOCK) void advantage_kernel(AdvArgs a, SourceDesc sd) {
    __shared__ AdvLds L;
    const int N = a.n_seq;

    // ---- per-sequence advantages + layout validation ----
    const int64_t gid = (int64_t)blockIdx.x * ADV_BLOCK + threadIdx.x;
    if (gid < N) {
        const int i = (int)gid;
        a.adv_seq[i] = seq_advantage(a, i);
        int s = 0;
        while (s + 1 < sd.n_src && i >= sd.seq_off[s + 1]) ++s;
        const int64_t so = a.src_tok_off[i];
        const int32_t ln = a.seq_len[i];
        if (ln <= 0 || ln > DC_MAX_SEQ_LEN) set_status(a.status, DC_ERR_ZERO_LENGTH_SEQ);
        else if (so < 0 || so + ln > sd.tokens[s]) set_status(a.status, DC_ERR_BAD_LAYOUT);
        else if (i + 1 < sd.seq_off[s + 1] && a.src_tok_off[i + 1] < so + ln) set_status(a.status, DC_ERR_BAD_LAYOUT);
    }
    if (gid <= a.n_groups) {
        const int g = (int)gid;
        const int32_t v = a.group_off[g];
        bool bad = v < 0 || v > N || (g == 0 && v != 0) || (g == a.n_groups && v != N);
        if (g < a.n_groups && a.group_off[g + 1] < v) bad = true;
        if (bad) set_status(a.status, DC_ERR_BAD_LAYOUT);
    }
    if (a.n_src == 0) return;                           // no per-token output requested

    // ---- which rollout shard / tile is mine ----
    int s = 0;
    while (s + 1 < a.n_src && (int)blockIdx.x >= a.tile_off[s + 1]) ++s;
    if ((int)blockIdx.x >= a.tile_off[a.n_src]) return; // workgroup only served the per-sequence part
    const int64_t shard_tokens = sd.tokens[s];
    const int64_t tile_begin = (int64_t)(blockIdx.x - a.tile_off[s]) * ADV_TILE;
    const int64_t tile_end = min(tile_begin + (int64_t)ADV_TILE, shard_tokens);
    const int seq_lo = sd.seq_off[s], seq_hi = sd.seq_off[s + 1];
    if (tile_begin >= tile_end || seq_lo >= seq_hi) return;
    const uint8_t* __restrict__ mask = a.mask[s];
    float* __restrict__ out = a.adv_tok[s];

    // first sequence that can reach into the tile: last i with src_tok_off[i] <= tile_begin
    int lo = seq_lo, hi = seq_hi;                       // first i with src_tok_off[i] > tile_begin
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a.src_tok_off[mid] <= tile_begin) lo = mid + 1; else hi = mid;
    }
    int seg_base = max(lo - 1, seq_lo);

    int64_t pass_begin = tile_begin;
    for (;;) {
        for (int k = threadIdx.x; k < ADV_NSEG; k += ADV_BLOCK) {
            const int64_t i = (int64_t)seg_base + k;
            int64_t st = INT64_MAX;
            int32_t ln = 0;
            float av = 0.0f;
            if (i < seq_hi) {
                st = a.src_tok_off[i];
                ln = a.seq_len[i];
                if (ln < 0) ln = 0;
                if (st < tile_end && st + ln > tile_begin) av = seq_advantage(a, (int)i);
            }
            L.start[k] = st; L.len[k] = ln; L.adv[k] = av;
        }
        __syncthreads();
        int n_all = 0;                                  // entries with start < tile_end
        {
            int l2 = 0, h2 = ADV_NSEG;
            while (l2 < h2) { const int mid = (l2 + h2) >> 1; if (L.start[mid] < tile_end) l2 = mid + 1; else h2 = mid; }
            n_all = l2;
        }
        const bool more = n_all > SEG_BATCH;
        const int64_t pass_end = more ? L.start[SEG_BATCH] : tile_end;

        constexpr int STEPS = ADV_TILE / 4 / ADV_BLOCK;  // 4-token chunks per lane
#pragma unroll
        for (int u = 0; u < STEPS; ++u) {
            const int64_t c0 = tile_begin + (int64_t)(threadIdx.x + u * ADV_BLOCK) * 4;
            if (c0 < pass_begin || c0 >= pass_end) continue;
            int l3 = 0, h3 = n_all;                     // largest k with start[k] <= c0
            while (l3 < h3) { const int mid = (l3 + h3) >> 1; if (L.start[mid] <= c0) l3 = mid + 1; else h3 = mid; }
            int k = l3 - 1;
            bool whole = false;
            if (k >= 0) {
                const int64_t st = L.start[k];
                whole = c0 + 4 <= st + L.len[k] && c0 + 4 <= tile_end;
            }
            if (whole) {
                const uint32_t mk = load4(mask + c0);
                const uint32_t av = __float_as_uint(L.adv[k]);
                u32x4 o;
                o.x = (mk & 0x000000FFu) ? av : 0u;
                o.y = (mk & 0x0000FF00u) ? av : 0u;
                o.z = (mk & 0x00FF0000u) ? av : 0u;
                o.w = (mk & 0xFF000000u) ? av : 0u;
                store16(out + c0, o);
            } else {
                for (int e = 0; e < 4; ++e) {
                    const int64_t tok = c0 + e;
                    if (tok >= tile_end) break;
                    while (k + 1 < n_all && L.start[k + 1] <= tok) ++k;
                    if (k >= 0) {
                        const int64_t st = L.start[k];
                        if (tok >= st && tok < st + L.len[k]) out[tok] = mask[tok] ? L.adv[k] : 0.0f;
                    }
                }
            }
        }
        if (!more) break;
        seg_base += SEG_BATCH;
        pass_begin = pass_end;
        __syncthreads();
    }
}

hipError_t launch_advantage(int32_t n_seq, const SourceDesc& src, const int64_t* d_src_tok_off,
                            const int32_t* d_seq_len, const float* d_reward, const int32_t* d_group_off,
                            int32_t n_groups, double eps, int32_t ddof,
                            const uint8_t* const* mask_base, float* d_adv_seq, float* const* adv_tok_base,
                            int32_t* d_status, hipStream_t st) {
    AdvArgs a;
    a.n_seq = n_seq; a.n_groups = n_groups; a.ddof = ddof; a.eps = eps;
    a.src_tok_off = d_src_tok_off; a.seq_len = d_seq_len; a.reward = d_reward; a.group_off = d_group_off;
    a.adv_seq = d_adv_seq; a.status = d_status;
    const bool per_token = adv_tok_base != nullptr;
    a.n_src = per_token ? src.n_src : 0;
    int64_t blocks = 0;
    for (int s = 0; s < DC_MAX_SRC_SHARDS; ++s) {
        a.tile_off[s] = (int32_t)blocks;
        a.mask[s] = nullptr; a.adv_tok[s] = nullptr;
        if (per_token && s < src.n_src) {
            a.mask[s] = mask_base[s]; a.adv_tok[s] = adv_tok_base[s];
            blocks += (src.tokens[s] + ADV_TILE - 1) / ADV_TILE;
        }
    }
    a.tile_off[DC_MAX_SRC_SHARDS] = (int32_t)blocks;
    for (int s = src.n_src; s <= DC_MAX_SRC_SHARDS; ++s) a.tile_off[s] = (int32_t)blocks;
    const int64_t need = ((int64_t)(n_seq > n_groups + 1 ? n_seq : n_groups + 1) + ADV_BLOCK - 1) / ADV_BLOCK;
    const int64_t grid = blocks > need ? blocks : need;
    if (grid == 0) return hipSuccess;
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(advantage_kernel, dim3((unsigned)grid), dim3(ADV_BLOCK), 0, st, a, src);
    return hipGetLastError();
}

}  // namespace dc
