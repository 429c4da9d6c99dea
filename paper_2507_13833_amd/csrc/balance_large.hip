// Algorithm 1 for more sequences than one workgroup's LDS holds (dc_balance_ws above DC_MAX_SEQ).
#include "balance_device.h"

namespace dc {

// N > DC_MAX_SEQ (up to DC_MAX_SEQ_LARGE): the same algorithm by one workgroup, with the
// index arrays of the sort in a caller-supplied workspace and the assignment fed in portions of
// DC_MAX_SEQ sorted items, staged into the LDS arrays the rounds read (lpt_rounds / lpt_rounds_wide as they are; the
// workers' keys, counts and loads are carried from portion to portion).  A slow path next to
// balance.hip's: every access to the index arrays is a global one.
struct BalanceLargeWs {
    int32_t* idx_a;        // [N] sort ping
    int32_t* idx_b;        // [N] sort pong
    int32_t* place;        // [N] by sorted position: worker << 16 | place inside its partition
};

// counting_pass with positions, digits and outputs outside the LDS.  Wave w owns the contiguous positions
// [w * per_wave, (w + 1) * per_wave); a first sweep counts per (digit, wave), a second one repeats the
// matching and hands out places from the scanned counters, which each wave advances as it goes (its
// positions are visited in order, so the order inside a digit stays the input order).
template <typename DigitFn, typename EmitFn>
__device__ __forceinline__ void counting_pass_large(BalLds& L, int N, DigitFn digit, EmitFn emit) {
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    const int per_wave = ((N + BAL_BLOCK - 1) / BAL_BLOCK) * WAVE;
    const int begin = w * per_wave, end = min(N, begin + per_wave);
    for (int i = tid; i < 256 * BAL_WAVES; i += BAL_BLOCK) L.cnt[i] = 0;
    __syncthreads();
    for (int sweep = 0; sweep < 2; ++sweep) {
        for (int base = begin; base < end; base += WAVE) {           // uniform over the wave
            const int pos = base + lane;
            const bool valid = pos < end;
            uint32_t d = 0;
            if (valid) d = digit(pos) & 0xFFu;
            const uint64_t valid_lanes = __builtin_amdgcn_ballot_w64(valid);
            uint32_t peers_lo = (uint32_t)valid_lanes, peers_hi = (uint32_t)(valid_lanes >> 32);
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const uint64_t bal = __builtin_amdgcn_ballot_w64(((d >> b) & 1u) != 0u);
                const uint32_t mine = (uint32_t)__builtin_amdgcn_sbfe((int)d, (unsigned)b, 1u);
                peers_lo &= ~((uint32_t)bal ^ mine);
                peers_hi &= ~((uint32_t)(bal >> 32) ^ mine);
            }
            const uint64_t peers = ((uint64_t)peers_hi << 32) | peers_lo;
            const int before = __popcll(peers & ((1ull << lane) - 1ull));
            const int leader = valid ? (__ffsll((long long)peers) - 1) : lane;
            uint32_t old = 0;
            if (valid && lane == leader) {                        // one lane per distinct digit
                uint32_t* c = &L.cnt[d * BAL_WAVES + w];
                old = *c;
                *c = old + (uint32_t)__popcll(peers);
            }
            old = (uint32_t)__shfl((int)old, leader, WAVE);
            if (sweep == 1 && valid) emit(pos, (int)(old + (uint32_t)before));
        }
        __syncthreads();
        if (sweep == 0) {   // exclusive scan of the 4096 counters in (digit, wave) order
            uint32_t c4[4], sum = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) { c4[q] = L.cnt[tid * 4 + q]; sum += c4[q]; }
            uint32_t tot;
            uint32_t run = block_excl_scan_add<uint32_t>(sum, L.tmp32, &tot);
#pragma unroll
            for (int q = 0; q < 4; ++q) { L.cnt[tid * 4 + q] = run; run += c4[q]; }
            __syncthreads();
        }
    }
}

__device__ __forceinline__ int32_t sane_len(int32_t s) { return (s <= 0 || s > DC_MAX_SEQ_LEN) ? 1 : s; }

__global__ __launch_bounds__(BAL_BLOCK) void balance_large_kernel(int32_t N, int32_t P, int32_t C,
                                                                  const int32_t* __restrict__ seq_len,
                                                                  int32_t* __restrict__ perm,
                                                                  int32_t* __restrict__ shard_seq_off,
                                                                  int32_t* __restrict__ shard_of_seq,
                                                                  int64_t* __restrict__ shard_load,
                                                                  BalanceLargeWs ws, int32_t* status) {
    __shared__ BalLds L;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;

    // ---- range of the lengths ----
    int32_t mx = 0, mn = INT32_MAX;
    bool bad = false;
    for (int i = tid; i < N; i += BAL_BLOCK) {
        const int32_t raw = seq_len[i], sl = sane_len(raw);
        bad = bad || sl != raw;
        mx = max(mx, sl);
        mn = min(mn, sl);
        ws.idx_a[i] = i;
    }
    if (bad) set_status(status, DC_ERR_ZERO_LENGTH_SEQ);
    for (int d = 32; d >= 1; d >>= 1) {
        mx = max(mx, __shfl_xor(mx, d, WAVE));
        mn = min(mn, __shfl_xor(mn, d, WAVE));
    }
    if (lane == 0) { L.red[w] = mx; L.red[BAL_WAVES + w] = mn; }
    __syncthreads();                                              // also: idx_a is written
    mx = 0; mn = INT32_MAX;
    for (int i = 0; i < BAL_WAVES; ++i) { mx = max(mx, L.red[i]); mn = min(mn, L.red[BAL_WAVES + i]); }
    const uint32_t range = (uint32_t)(mx - mn);
    const int nbits = 32 - __clz(range | 1u);
    const int passes = range == 0 ? 0 : (nbits + 7) / 8;

    // ---- a) stable radix sort of the indices by (mx - len) ascending ----
    int32_t* src = ws.idx_a;
    int32_t* dst = ws.idx_b;
    for (int pass = 0; pass < passes; ++pass) {
        const int shift = pass * 8;
        counting_pass_large(L, N,
                            [&](int pos) { return ((uint32_t)(mx - sane_len(seq_len[src[pos]]))) >> shift; },
                            [&](int pos, int out) { dst[out] = src[pos]; });
        __threadfence_block();
        __syncthreads();
        int32_t* t = src; src = dst; dst = t;
    }
    const int32_t* sorted = src;                                  // I of Algorithm 1

    // ---- b) the assignment, DC_MAX_SEQ sorted items at a time ----
    int32_t* worker_count = reinterpret_cast<int32_t*>(L.cnt) + WCOUNT_AT;
    int32_t* part_off = reinterpret_cast<int32_t*>(L.cnt) + PART_OFF_AT;
    LptCarry carry = lpt_fresh(P, C);                             // up to 64 workers: wave 0's lanes keep them
    WideCarry wide = wide_fresh(P, C);                            // more: thread k keeps worker k
    for (int c0 = 0; c0 < N; c0 += DC_MAX_SEQ) {
        const int n = min(DC_MAX_SEQ, N - c0);
        for (int t = tid; t < n; t += BAL_BLOCK) {
            L.keys[t] = sane_len(seq_len[sorted[c0 + t]]);
            L.idx_a[t] = (uint16_t)t;                             // the portion is in order already
        }
        __syncthreads();
        if (P > WAVE) {
            lpt_rounds_wide_portion(L, n, P, C, L.idx_a, L.idx_b, wide);
        } else if (w == 0) {
            if (P <= 16) lpt_rounds<16>(n, P, C, L.keys, L.idx_a, mx, L.idx_b, 0, L.spare, worker_count, shard_load, carry);
            else if (P <= 32) lpt_rounds<32>(n, P, C, L.keys, L.idx_a, mx, L.idx_b, 0, L.spare, worker_count, shard_load, carry);
            else lpt_rounds<64>(n, P, C, L.keys, L.idx_a, mx, L.idx_b, 0, L.spare, worker_count, shard_load, carry);
        }
        __syncthreads();
        for (int t = tid; t < n; t += BAL_BLOCK)                  // keys[t]: the worker that took item t of the portion
            ws.place[c0 + t] = (L.keys[t] << 16) | (int32_t)L.idx_b[t];
        __syncthreads();
    }
    if (P > WAVE) {
        lpt_wide_finish(L, N, P, wide, shard_seq_off, shard_load);
    } else if (w == 0) {                                          // start of every P_k inside perm
        const int32_t c = worker_count[lane];
        const int32_t inc = (int32_t)wave_incl_scan_add_u32((uint32_t)c);
        part_off[lane] = inc - c;
        if (lane < P) shard_seq_off[lane] = inc - c;
        if (lane == 0) shard_seq_off[P] = N;
    }
    __threadfence_block();
    __syncthreads();

    // ---- c) lay out P_0, P_1, ... each in insertion order ----
    for (int t = tid; t < N; t += BAL_BLOCK) {
        const int u = sorted[t];
        const int32_t pl = ws.place[t];
        const int k = min((int)((uint32_t)pl >> 16), P - 1);      // (every item is placed: P * C >= N; no index leaves
        shard_of_seq[u] = k;                                      //  the arrays whatever the words hold)
        perm[min(part_off[k] + (pl & 0xFFFF), N - 1)] = u;
    }
}

hipError_t launch_balance_large(int32_t n_seq, int32_t n_shards, int32_t cap_eff, const int32_t* d_seq_len,
                                int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                                int64_t* d_shard_load, void* d_ws, int32_t* d_status, hipStream_t st) {
    BalanceLargeWs ws;
    const size_t n = ((size_t)n_seq + 63) & ~(size_t)63;           // each array starts on a 256-byte boundary
    ws.idx_a = static_cast<int32_t*>(d_ws);
    ws.idx_b = ws.idx_a + n;
    ws.place = ws.idx_b + n;
    hipLaunchKernelGGL(balance_large_kernel, dim3(1), dim3(BAL_BLOCK), 0, st, n_seq, n_shards, cap_eff, d_seq_len,
                       d_perm, d_shard_seq_off, d_shard_of_seq, d_shard_load, ws, d_status);
    return hipGetLastError();
}

}  // namespace dc
