// Algorithm 1, Constrained LPT Load Balancing (Sec. 6 "Load Balancing").
//
// One workgroup, everything in LDS (N <= DC_MAX_SEQ, P <= 64):
//   a) stable LSD radix sort of the sequence indices by descending length
//      (8-bit digits of max_len - len, only as many passes as the length range
//      needs; ranks inside a wave by ballot matching, across waves by a scan of
//      per-wave digit counters);
//   b) the assignment loop on wave 0, lane k = worker k.  A lane keeps its worker's
//      item count and a 32-bit key (load - base) << 6 | k, all-ones when the worker
//      is full; "pop the minimum that is not full" is one DPP min-reduction over
//      the 64 keys.  Loads of workers that are not full never differ by more than
//      the longest sequence, so rebasing the keys when the minimum grows large keeps
//      them in 32 bits for any total load;
//   c) all lanes lay the P_k out one after the other (insertion order).
#include "dc_device.h"
#include "dc_internal.h"

namespace dc {

constexpr int BAL_BLOCK = 1024;
constexpr int BAL_WAVES = BAL_BLOCK / WAVE;
constexpr int BAL_ROUNDS = DC_MAX_SEQ / BAL_BLOCK;       // 64-item rounds per wave at the size limit
constexpr uint32_t KEY_FULL = 0xFFFFFFFFu;

struct BalLds {
    int32_t  keys[DC_MAX_SEQ];            // sequence lengths (sanitised)
    uint16_t idx_a[DC_MAX_SEQ];           // sort ping
    uint16_t idx_b[DC_MAX_SEQ];           // sort pong; after the sort: rank of step t inside its worker
    uint32_t cnt[256 * BAL_WAVES];        // [digit][wave] counters; after the sort: worker of step t (bytes)
    int64_t  load[DC_MAX_SHARDS];
    int32_t  off[DC_MAX_SHARDS + 1];
    int32_t  red[2 * BAL_WAVES];
    uint32_t tmp32[16];
};

__device__ __forceinline__ uint32_t dpp_min_step(uint32_t v, uint32_t moved) { return moved < v ? moved : v; }

// Minimum of v over the 64 lanes, returned to every lane (uniform).
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    // lanes without a source keep their own value (old = v), which is harmless for min
    v = dpp_min_step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x111, 0xF, 0xF, false));  // row_shr:1
    v = dpp_min_step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x112, 0xF, 0xF, false));  // row_shr:2
    v = dpp_min_step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x114, 0xF, 0xF, false));  // row_shr:4
    v = dpp_min_step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x118, 0xF, 0xF, false));  // row_shr:8
    v = dpp_min_step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x142, 0xF, 0xF, false));  // row_bcast:15
    v = dpp_min_step(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x143, 0xF, 0xF, false));  // row_bcast:31
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

__global__ __launch_bounds__(BAL_BLOCK) void balance_kernel(int32_t N, int32_t P, int32_t C,
                                                            const int32_t* __restrict__ seq_len,
                                                            int32_t* __restrict__ perm,
                                                            int32_t* __restrict__ shard_seq_off,
                                                            int32_t* __restrict__ shard_of_seq,
                                                            int64_t* __restrict__ shard_load,
                                                            int32_t* status) {
    __shared__ BalLds L;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;

    // ---- load lengths, range ----
    int32_t mx = 0, mn = INT32_MAX;
    for (int i = tid; i < N; i += BAL_BLOCK) {
        int32_t s = seq_len[i];
        if (s <= 0 || s > DC_MAX_SEQ_LEN) { set_status(status, DC_ERR_ZERO_LENGTH_SEQ); s = 1; }
        L.keys[i] = s;
        mx = max(mx, s);
        mn = min(mn, s);
    }
    for (int d = 32; d >= 1; d >>= 1) {
        mx = max(mx, __shfl_xor(mx, d, WAVE));
        mn = min(mn, __shfl_xor(mn, d, WAVE));
    }
    if (lane == 0) { L.red[w] = mx; L.red[BAL_WAVES + w] = mn; }
    __syncthreads();
    mx = 0; mn = INT32_MAX;
    for (int i = 0; i < BAL_WAVES; ++i) { mx = max(mx, L.red[i]); mn = min(mn, L.red[BAL_WAVES + i]); }
    const uint32_t range = N > 0 ? (uint32_t)(mx - mn) : 0u;
    const int nbits = 32 - __clz(range | 1u);
    const int passes = range == 0 ? 0 : (nbits + 7) / 8;

    // ---- a) radix sort of indices by (mx - len) ascending, stable ----
    const int rounds = (N + BAL_BLOCK - 1) / BAL_BLOCK;           // <= BAL_ROUNDS
    const int wave_base = w * rounds * WAVE;                      // wave w owns positions [wave_base, +rounds*64)
    for (int i = tid; i < N; i += BAL_BLOCK) L.idx_a[i] = (uint16_t)i;
    uint16_t* src = L.idx_a;
    uint16_t* dst = L.idx_b;
    __syncthreads();
    for (int pass = 0; pass < passes; ++pass) {
        const int shift = pass * 8;
        for (int i = tid; i < 256 * BAL_WAVES; i += BAL_BLOCK) L.cnt[i] = 0;
        __syncthreads();
        uint32_t packed[BAL_ROUNDS];                              // digit << 16 | rank before me in my wave
#pragma unroll
        for (int r = 0; r < BAL_ROUNDS; ++r) {
            packed[r] = 0;
            if (r < rounds) {                                     // uniform
                const int pos = wave_base + r * WAVE + lane;
                const bool valid = pos < N;
                uint32_t d = 0;
                if (valid) d = (((uint32_t)(mx - L.keys[src[pos]])) >> shift) & 0xFFu;
                uint64_t peers = __ballot(valid);
#pragma unroll
                for (int b = 0; b < 8; ++b) {
                    const uint64_t bal = __ballot(valid && ((d >> b) & 1u));
                    peers &= ((d >> b) & 1u) ? bal : ~bal;
                }
                const uint64_t lt = (1ull << lane) - 1ull;
                const int before = __popcll(peers & lt);
                const int leader = valid ? (__ffsll((long long)peers) - 1) : lane;
                uint32_t old = 0;
                if (valid && lane == leader) {                    // one lane per distinct digit
                    uint32_t* c = &L.cnt[d * BAL_WAVES + w];
                    old = *c;
                    *c = old + (uint32_t)__popcll(peers);
                }
                old = (uint32_t)__shfl((int)old, leader, WAVE);
                packed[r] = (d << 16) | (old + (uint32_t)before);
            }
        }
        __syncthreads();
        {   // exclusive scan of the 4096 counters in (digit, wave) order
            uint32_t c4[4], s = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) { c4[q] = L.cnt[tid * 4 + q]; s += c4[q]; }
            uint32_t tot;
            uint32_t run = block_excl_scan_add<uint32_t>(s, L.tmp32, &tot);
#pragma unroll
            for (int q = 0; q < 4; ++q) { L.cnt[tid * 4 + q] = run; run += c4[q]; }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < BAL_ROUNDS; ++r) {
            if (r < rounds) {
                const int pos = wave_base + r * WAVE + lane;
                if (pos < N) {
                    const uint32_t d = packed[r] >> 16, rk = packed[r] & 0xFFFFu;
                    dst[L.cnt[d * BAL_WAVES + w] + rk] = src[pos];
                }
            }
        }
        __syncthreads();
        uint16_t* t = src; src = dst; dst = t;
    }
    // src: sorted indices.  dst: free -> rank inside worker per step.  cnt: free -> worker per step.
    const uint16_t* sorted = src;
    uint16_t* step_rank = dst;
    uint8_t* step_worker = reinterpret_cast<uint8_t*>(L.cnt);     // 16 KiB >= DC_MAX_SEQ bytes

    // ---- b) assignment loop, wave 0 ----
    if (w == 0) {
        uint32_t key = lane < P ? (uint32_t)lane : KEY_FULL;
        if (C == 0) key = KEY_FULL;
        int32_t count = 0;
        int64_t load = 0;
        for (int base = 0; base < N; base += WAVE) {
            int32_t my_s = 0;
            if (base + lane < N) my_s = L.keys[sorted[base + lane]];
            const int n_here = min(WAVE, N - base);
            for (int q = 0; q < n_here; ++q) {
                const uint32_t s = (uint32_t)__builtin_amdgcn_readlane(my_s, q);
                const uint32_t m = wave_min_u32(key);
                const int k = (int)(m & 63u);
                if (lane == k) {
                    step_rank[base + q] = (uint16_t)count;
                    step_worker[base + q] = (uint8_t)k;
                    count += 1;
                    load += s;
                    key = (count == C) ? KEY_FULL : key + (s << 6);
                }
                if (m >= 0x40000000u) {                           // rebase: subtract the minimum load
                    const uint32_t sub = m & ~63u;
                    if (key != KEY_FULL) key -= sub;
                }
            }
        }
        if (lane < P) { L.load[lane] = load; shard_load[lane] = load; }
        const int32_t inc = wave_incl_scan_add<int32_t>(lane < P ? count : 0);
        if (lane < P) L.off[lane + 1] = inc;
        if (lane == 0) L.off[0] = 0;
    }
    __syncthreads();

    // ---- c) lay out P_0, P_1, ... ----
    for (int t = tid; t < N; t += BAL_BLOCK) {
        const int k = step_worker[t];
        const int u = sorted[t];
        perm[L.off[k] + step_rank[t]] = u;
        shard_of_seq[u] = k;
    }
    if (tid <= P) shard_seq_off[tid] = L.off[tid];
}

hipError_t launch_balance(int32_t n_seq, int32_t n_shards, int32_t cap_eff, const int32_t* d_seq_len,
                          int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                          int64_t* d_shard_load, int32_t* d_status, hipStream_t st) {
    hipLaunchKernelGGL(balance_kernel, dim3(1), dim3(BAL_BLOCK), 0, st, n_seq, n_shards, cap_eff, d_seq_len,
                       d_perm, d_shard_seq_off, d_shard_of_seq, d_shard_load, d_status);
    return hipGetLastError();
}

}  // namespace dc
