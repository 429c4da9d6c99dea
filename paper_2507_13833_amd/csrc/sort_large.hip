// Argsort of the sequence lengths for more sequences than one workgroup's LDS holds (Algorithm 1's first
// statement above DC_MAX_SEQ sequences): a stable LSD radix sort of the sequence indices by descending
// length over MANY workgroups, three passes of 8 bits (lengths are at most 2^24), each pass three launches:
//   count    every workgroup takes a tile of SORT_TILE positions and counts its digits;
//   scan     workgroup d turns the counts of digit d into running sums over the tiles and notes the digit's total;
//   scatter  every workgroup scans the 256 totals (where each digit starts), ranks its tile again, stably (wave
//            by wave, lanes with equal digits matched by ballots), and moves the indices; the last pass also
//            writes the lengths in sorted order.
// No workgroup ever waits for another inside a launch; the launches of a pass order them.
#include "dc_device.h"
#include "dc_internal.h"

namespace dc {

constexpr int SORT_BLOCK = 256;
constexpr int SORT_WAVES = SORT_BLOCK / WAVE;
constexpr int SORT_PER_WAVE = 256;                        // consecutive positions of one wave
constexpr int SORT_TILE = SORT_WAVES * SORT_PER_WAVE;     // positions of one workgroup
constexpr int SORT_LEN_BITS = 24;
static_assert((1 << SORT_LEN_BITS) >= DC_MAX_SEQ_LEN, "three 8-bit passes cover every length");

struct SortArgs {
    int32_t        n;
    int32_t        n_tiles;
    int32_t        shift;             // 0, 8, 16
    const int32_t* seq_len;
    const int32_t* src;               // indices in the order of the pass before (null: the identity)
    int32_t*       dst;
    uint32_t*      counts;            // [256 * n_tiles], digit-major
    uint32_t*      totals;            // [256] items per digit
    int32_t*       len_out;           // last pass: the lengths in the order of dst (else null)
    int32_t*       status;            // first pass: DC_ERR_ZERO_LENGTH_SEQ for a length outside (0, 2^24] (else null)
};

// Key of a sequence: ascending keys = descending lengths; lengths outside (0, 2^24] count as 1, as everywhere.
__device__ __forceinline__ int32_t sort_len(int32_t len) { return (len <= 0 || len > DC_MAX_SEQ_LEN) ? 1 : len; }
__device__ __forceinline__ uint32_t sort_key(int32_t len) { return (uint32_t)(DC_MAX_SEQ_LEN - sort_len(len)); }

// For the wave's positions base .. base + 63 (valid below n_end): my digit, the lanes of this step that hold the
// same digit, and how many of them stand before me.
__device__ __forceinline__ void match_digits(bool valid, uint32_t d, int lane, uint64_t* peers_out, int* before_out) {
    const uint64_t valid_lanes = __builtin_amdgcn_ballot_w64(valid);
    uint32_t peers_lo = (uint32_t)valid_lanes, peers_hi = (uint32_t)(valid_lanes >> 32);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const uint64_t bal = __builtin_amdgcn_ballot_w64(((d >> b) & 1u) != 0u);
        const uint32_t mine = (uint32_t)__builtin_amdgcn_sbfe((int)d, (unsigned)b, 1u);      // all ones if my bit is set
        peers_lo &= ~((uint32_t)bal ^ mine);
        peers_hi &= ~((uint32_t)(bal >> 32) ^ mine);
    }
    const uint64_t peers = ((uint64_t)peers_hi << 32) | peers_lo;
    *peers_out = peers;
    *before_out = __popcll(peers & ((1ull << lane) - 1ull));
}

__global__ __launch_bounds__(SORT_BLOCK) void sort_count_kernel(SortArgs a) {
    __shared__ uint32_t cnt[256];
    const int tid = threadIdx.x;
    cnt[tid] = 0;
    __syncthreads();
    const int begin = blockIdx.x * SORT_TILE, end = min(a.n, begin + SORT_TILE);
    for (int pos = begin + tid; pos < end; pos += SORT_BLOCK) {
        const int32_t i = a.src ? a.src[pos] : pos;
        const int32_t raw = a.seq_len[min(max(i, 0), a.n - 1)];
        if (a.status && raw != sort_len(raw)) set_status(a.status, DC_ERR_ZERO_LENGTH_SEQ);
        const uint32_t d = (sort_key(raw) >> a.shift) & 0xFFu;
        atomicAdd(&cnt[d], 1u);                                   // (only the totals matter here)
    }
    __syncthreads();
    a.counts[(size_t)tid * a.n_tiles + blockIdx.x] = cnt[tid];
}

// Workgroup d: exclusive scan of counts[d][0 .. n_tiles) in place; totals[d] = their sum.
__global__ __launch_bounds__(SORT_BLOCK) void sort_scan_kernel(uint32_t* counts, uint32_t* totals, int32_t n_tiles) {
    __shared__ uint32_t tmp[SORT_WAVES];
    const int tid = threadIdx.x;
    uint32_t* row = counts + (size_t)blockIdx.x * n_tiles;
    uint32_t carry = 0;
    for (int base = 0; base < n_tiles; base += SORT_BLOCK) {      // (uniform)
        const int i = base + tid;
        const uint32_t c = i < n_tiles ? row[i] : 0u;
        uint32_t all;
        const uint32_t before = block_excl_scan_add<uint32_t>(c, tmp, &all);
        if (i < n_tiles) row[i] = carry + before;
        carry += all;
    }
    if (tid == 0) totals[blockIdx.x] = carry;
}

__global__ __launch_bounds__(SORT_BLOCK) void sort_scatter_kernel(SortArgs a) {
    constexpr int PITCH = SORT_WAVES + 1;                         // odd: the digits' rows start in different LDS banks
    __shared__ uint32_t cnt[256 * PITCH];                         // [digit][wave]: first counts, then the wave's next place
    __shared__ uint32_t tmp[SORT_WAVES];
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    uint32_t n_all;
    const uint32_t digit_start = block_excl_scan_add<uint32_t>(a.totals[tid], tmp, &n_all);      // tid = digit
    for (int i = tid; i < 256 * PITCH; i += SORT_BLOCK) cnt[i] = 0;
    __syncthreads();
    const int begin = blockIdx.x * SORT_TILE + w * SORT_PER_WAVE, end = min(a.n, begin + SORT_PER_WAVE);
    for (int sweep = 0; sweep < 2; ++sweep) {
        for (int base = begin; base < end; base += WAVE) {       // uniform over the wave; positions in order
            const int pos = base + lane;
            const bool valid = pos < end;
            int32_t i = 0, len = 1;
            uint32_t d = 0;
            if (valid) {
                i = a.src ? a.src[pos] : pos;
                len = sort_len(a.seq_len[min(max(i, 0), a.n - 1)]);
                d = (sort_key(len) >> a.shift) & 0xFFu;
            }
            uint64_t peers;
            int before;
            match_digits(valid, d, lane, &peers, &before);
            const int leader = valid ? (__ffsll((long long)peers) - 1) : lane;
            uint32_t old = 0;
            if (valid && lane == leader) {                        // one lane per distinct digit
                uint32_t* c = &cnt[d * PITCH + w];
                old = *c;
                *c = old + (uint32_t)__popcll(peers);
            }
            old = (uint32_t)__shfl((int)old, leader, WAVE);
            if (sweep == 1 && valid) {
                const uint32_t out = min(old + (uint32_t)before, (uint32_t)(a.n - 1));
                a.dst[out] = i;
                if (a.len_out) a.len_out[out] = len;
            }
        }
        __syncthreads();
        if (sweep == 0) {
            // the wave's first place for every digit: where the digit starts for this tile, plus the waves before
            const uint32_t start = digit_start + a.counts[(size_t)tid * a.n_tiles + blockIdx.x];
            uint32_t run = start;
#pragma unroll
            for (int q = 0; q < SORT_WAVES; ++q) { const uint32_t c = cnt[tid * PITCH + q]; cnt[tid * PITCH + q] = run; run += c; }
            __syncthreads();
        }
    }
}

// Bytes of the (digit, tile) table for n sequences.
size_t sort_large_table_bytes(int32_t n_seq) {
    const size_t tiles = ((size_t)n_seq + SORT_TILE - 1) / SORT_TILE;
    return 256 * (tiles + 1) * sizeof(uint32_t);                  // the (digit, tile) counts, then the digits' totals
}

// d_idx_a, d_idx_b, d_sorted_len: arrays of n_seq int32; d_counts: sort_large_table_bytes(n_seq).  The passes go
// identity -> b, b -> a, a -> b: the sorted indices end in d_idx_b, their lengths in d_sorted_len, d_idx_a is free again.
hipError_t launch_sort_large(int32_t n_seq, const int32_t* d_seq_len, int32_t* d_idx_a, int32_t* d_idx_b,
                             int32_t* d_sorted_len, uint32_t* d_counts, int32_t* d_status, hipStream_t st) {
    SortArgs a;
    a.n = n_seq;
    a.n_tiles = (n_seq + SORT_TILE - 1) / SORT_TILE;
    a.seq_len = d_seq_len;
    a.counts = d_counts;
    a.totals = d_counts + (size_t)256 * a.n_tiles;
    const int32_t* src = nullptr;
    int32_t* dst = d_idx_b;
    for (int pass = 0; pass < SORT_LEN_BITS / 8; ++pass) {
        a.shift = 8 * pass;
        a.src = src;
        a.dst = dst;
        a.status = pass == 0 ? d_status : nullptr;
        a.len_out = pass == SORT_LEN_BITS / 8 - 1 ? d_sorted_len : nullptr;
        hipLaunchKernelGGL(sort_count_kernel, dim3((unsigned)a.n_tiles), dim3(SORT_BLOCK), 0, st, a);
        hipLaunchKernelGGL(sort_scan_kernel, dim3(256), dim3(SORT_BLOCK), 0, st, a.counts, a.totals, a.n_tiles);
        hipLaunchKernelGGL(sort_scatter_kernel, dim3((unsigned)a.n_tiles), dim3(SORT_BLOCK), 0, st, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        src = dst;
        dst = dst == d_idx_b ? d_idx_a : d_idx_b;
    }
    return hipSuccess;                                            // (src == d_idx_b: the order of the last pass)
}

}  // namespace dc
