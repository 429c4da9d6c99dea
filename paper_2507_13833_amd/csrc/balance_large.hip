// Algorithm 1 for more sequences than one workgroup's LDS holds (dc_balance_ws above DC_MAX_SEQ).
#include "balance_device.h"

namespace dc {

// N > DC_MAX_SEQ (up to DC_MAX_SEQ_LARGE), three stages in stream order:
//   1. launch_sort_large (sort_large.hip): the indices by descending length, and the lengths in that order, by
//      many workgroups;
//   2. balance_large_kernel: the assignment by ONE workgroup, fed DC_MAX_SEQ sorted items at a time, staged into the
//      LDS arrays the rounds read (lpt_rounds / lpt_rounds_wide as they are; the workers' keys, counts and loads are
//      carried from portion to portion); it leaves one word per sorted item: worker << 16 | place in its partition;
//   3. layout_large_kernel: perm and shard_of_seq from those words, by many workgroups.
// The printed algorithm (N == P * C) on 16, 32 or 64 workers with lengths below 2^16 runs lpt_rounds_packed on each
// portion instead; every partition's place in perm is known beforehand then (P_k starts at k * C), and stage 2 leaves,
// per place in perm, the sorted position of the item that stands there.
struct BalanceLargeWs {
    const int32_t* sorted;      // [N] I of Algorithm 1
    const int32_t* sorted_len;  // [N] S[I[t]]
    int32_t*       place;       // [N] by sorted position; packed rounds: by place in perm
};

// Both kernels take the same decision from the same words.
__device__ __forceinline__ bool packed_rounds_apply(int32_t N, int32_t P, int32_t C, int32_t longest) {
    return (P == 16 || P == 32 || P == 64) && (int64_t)P * C == N && (uint32_t)longest <= PACKED_MAX_LEN;
}

// Row length of a worker inside the LDS words that idx_a and idx_b span: odd, so that the rows start in different banks.
__device__ __forceinline__ int portion_pitch(int P) { return (((DC_MAX_SEQ + PLACE_PAD) / P) - 1) | 1; }

template <int WIDTH>
__device__ __forceinline__ void packed_portions(BalLds& L, int32_t N, int32_t P, int32_t C, int32_t mx,
                                                int32_t* __restrict__ shard_seq_off, int64_t* __restrict__ shard_load,
                                                const BalanceLargeWs& ws) {
    static_assert(offsetof(BalLds, idx_b) == offsetof(BalLds, idx_a) + sizeof(uint16_t) * (DC_MAX_SEQ + PLACE_PAD) &&
                  offsetof(BalLds, idx_a) % 4 == 0, "the two index arrays are one run of words");
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    uint32_t* const items = reinterpret_cast<uint32_t*>(L.keys);
    uint32_t* const rows = reinterpret_cast<uint32_t*>(L.idx_a);
    int32_t* const worker_count = reinterpret_cast<int32_t*>(L.cnt) + WCOUNT_AT;      // [64] after a portion
    int32_t* const count_before = worker_count + WAVE;                                // [64] before it
    int32_t* const placed = reinterpret_cast<int32_t*>(L.cnt) + PLACED_AT;
    const int pitch = portion_pitch(P);
    PackedCarry carry = packed_fresh(P, C);
    int c0 = 0;
    while (c0 < N) {                                              // (uniform)
        const int n = min(DC_MAX_SEQ, N - c0);
        for (int t = tid; t < n + PLACE_PAD; t += BAL_BLOCK)      // length << 16 | index inside the portion; zeros behind
            items[t] = t < n ? ((uint32_t)ws.sorted_len[c0 + t] << 16) | (uint32_t)t : 0u;
        __syncthreads();
        if (w == 0) {
            count_before[lane] = carry.count;
            const int done = lpt_rounds_packed<WIDTH, true>(n, P, C, items, mx, rows, pitch, reinterpret_cast<uint32_t*>(L.spare),
                                                            worker_count, shard_load, &carry, pitch);
            if (lane == 0) *placed = done;
        }
        __syncthreads();
        // empty the rows: worker k's items number count_before[k] .. worker_count[k] - 1 stand in perm from k * C on
        for (int k = w; k < P; k += BAL_WAVES) {
            const int first = count_before[k], got = min(worker_count[k] - first, pitch);
            for (int j = lane; j < got; j += WAVE) {
                const int at = k * C + first + j;
                if (at < N) ws.place[at] = c0 + (int32_t)(rows[k * pitch + j] & 0xFFFFu);
            }
        }
        const int done = *placed;
        __syncthreads();
        if (done <= 0) break;                                     // (cannot happen: an open worker always takes an item)
        c0 += done;
    }
    if (tid < P) shard_seq_off[tid] = tid * C;
    if (tid == 0) shard_seq_off[P] = N;
}

__global__ __launch_bounds__(BAL_BLOCK) void balance_large_kernel(int32_t N, int32_t P, int32_t C,
                                                                  int32_t* __restrict__ shard_seq_off,
                                                                  int64_t* __restrict__ shard_load,
                                                                  BalanceLargeWs ws) {
    __shared__ BalLds L;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    const int32_t mx = ws.sorted_len[0];                          // the longest sequence comes first

    if (packed_rounds_apply(N, P, C, mx)) {                       // (uniform)
        if (P == 16) packed_portions<16>(L, N, P, C, mx, shard_seq_off, shard_load, ws);
        else if (P == 32) packed_portions<32>(L, N, P, C, mx, shard_seq_off, shard_load, ws);
        else packed_portions<64>(L, N, P, C, mx, shard_seq_off, shard_load, ws);
        return;
    }

    int32_t* worker_count = reinterpret_cast<int32_t*>(L.cnt) + WCOUNT_AT;
    LptCarry carry = lpt_fresh(P, C);                             // up to 64 workers: wave 0's lanes keep them
    WideCarry wide = wide_fresh(P, C);                            // more: thread k keeps worker k
    for (int c0 = 0; c0 < N; c0 += DC_MAX_SEQ) {
        const int n = min(DC_MAX_SEQ, N - c0);
        for (int t = tid; t < n; t += BAL_BLOCK) {
            L.keys[t] = ws.sorted_len[c0 + t];
            L.idx_a[t] = (uint16_t)t;                             // the portion is in order already
        }
        __syncthreads();
        if (P > WAVE) {
            if ((uint32_t)mx <= PACKED_MAX_LEN) lpt_rounds_wide32_portion(L, n, P, C, L.idx_a, L.idx_b, wide);
            else lpt_rounds_wide_portion(L, n, P, C, L.idx_a, L.idx_b, wide);
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
        if (lane < P) shard_seq_off[lane] = inc - c;
        if (lane == 0) shard_seq_off[P] = N;
    }
}

// P_0, P_1, ... each in insertion order.
__global__ __launch_bounds__(256) void layout_large_kernel(int32_t N, int32_t P, int32_t C,
                                                           const int32_t* __restrict__ sorted,
                                                           const int32_t* __restrict__ sorted_len,
                                                           const int32_t* __restrict__ place,
                                                           const int32_t* __restrict__ shard_seq_off,
                                                           int32_t* __restrict__ perm, int32_t* __restrict__ shard_of_seq) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= N) return;
    if (packed_rounds_apply(N, P, C, sorted_len[0])) {            // place[q]: sorted position of the item at perm[q]
        const int u = min(max(sorted[min(max(place[t], 0), N - 1)], 0), N - 1);
        perm[t] = u;
        shard_of_seq[u] = t / C;
        return;
    }
    const int u = min(max(sorted[t], 0), N - 1);
    const int32_t pl = place[t];
    const int k = min((int)((uint32_t)pl >> 16), P - 1);          // (every item is placed: P * C >= N; no index leaves
    shard_of_seq[u] = k;                                          //  the arrays whatever the words hold)
    perm[min(max(shard_seq_off[k] + (pl & 0xFFFF), 0), N - 1)] = u;
}

hipError_t launch_balance_large(int32_t n_seq, int32_t n_shards, int32_t cap_eff, const int32_t* d_seq_len,
                                int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                                int64_t* d_shard_load, void* d_ws, int32_t* d_status, hipStream_t st) {
    const size_t n = ((size_t)n_seq + 63) & ~(size_t)63;           // each array starts on a 256-byte boundary
    int32_t* idx_a = static_cast<int32_t*>(d_ws);
    int32_t* idx_b = idx_a + n;
    int32_t* sorted_len = idx_b + n;
    uint32_t* counts = reinterpret_cast<uint32_t*>(sorted_len + n);
    hipError_t e = launch_sort_large(n_seq, d_seq_len, idx_a, idx_b, sorted_len, counts, d_status, st);
    if (e != hipSuccess) return e;
    BalanceLargeWs ws;
    ws.sorted = idx_b;
    ws.sorted_len = sorted_len;
    ws.place = idx_a;                                             // (the source of the sort's last pass: free again)
    hipLaunchKernelGGL(balance_large_kernel, dim3(1), dim3(BAL_BLOCK), 0, st, n_seq, n_shards, cap_eff,
                       d_shard_seq_off, d_shard_load, ws);
    hipLaunchKernelGGL(layout_large_kernel, dim3((unsigned)((n_seq + 255) / 256)), dim3(256), 0, st, n_seq, n_shards, cap_eff,
                       ws.sorted, ws.sorted_len, ws.place, d_shard_seq_off, d_perm, d_shard_of_seq);
    return hipGetLastError();
}

}  // namespace dc
