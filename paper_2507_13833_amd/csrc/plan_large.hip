// The plan of the packed training layout for more slots than one workgroup's LDS holds
// (DC_MAX_SEQ < N <= DC_MAX_SEQ_LARGE): plan_kernel's four steps by one workgroup, with the dense prefix
// of the slot lengths and the per-word tables in the workspace and the loops over N in steps of
// 1024 slots with a carry.  Only the bitmaps (first "sequence seen", then "slot opens a micro-batch") and
// the shard tables stay in the LDS.  A slow path: every probe of the prefix is a global access.
#include "dc_device.h"
#include "dc_internal.h"
#include "dc_lanes.h"

namespace dc {

constexpr int PLANL_BLOCK = 1024;
constexpr int PLANL_WAVES = PLANL_BLOCK / WAVE;

struct PlanLargeLds {
    uint32_t bits[DC_MAX_SEQ_LARGE / 32];   // one bit per sequence / per slot
    int64_t  shard_base[DC_MAX_SHARDS + 1]; // aligned token offset of each shard
    int32_t  shard_off[DC_MAX_SHARDS + 1];  // copy of shard_seq_off
    int64_t  tmp64[16];
    int32_t  tmp32[16];
    int32_t  ok;
};

// Exclusive max-scan over the workgroup (identity -1) and the maximum of all values.
__device__ __forceinline__ int32_t block_excl_scan_max_total(int32_t v, int32_t* tmp, int32_t* total) {
    const int lane = lane_id(), w = threadIdx.x / WAVE, nw = blockDim.x / WAVE;
    const int32_t inc = wave_incl_scan_max(v);
    if (lane == WAVE - 1) tmp[w] = inc;
    __syncthreads();
    const int32_t upto = wave_incl_scan_max(lane < nw ? tmp[lane] : -1);      // (lane i: the waves up to wave i)
    const int32_t base = wave_read_lane(wave_shift_up1(upto, -1), w);
    const int32_t up = wave_shift_up1(inc, -1);
    __syncthreads();
    *total = wave_read_lane(upto, WAVE - 1);
    return max(base, up);
}

__global__ __launch_bounds__(PLANL_BLOCK) void plan_large_kernel(PlanArgs a) {
    __shared__ PlanLargeLds L;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    const int N = a.n_seq, P = a.n_shards;
    const int n_words = (N + 31) / 32;

    for (int i = tid; i < n_words; i += PLANL_BLOCK) L.bits[i] = 0;
    if (tid == 0) L.ok = 1;
    __syncthreads();
    for (int p = tid; p <= P; p += PLANL_BLOCK) {
        const int32_t v = a.shard_seq_off[p];
        L.shard_off[p] = v;
        bool bad = v < 0 || v > N || (p == 0 && v != 0) || (p == P && v != N);
        if (p < P && a.shard_seq_off[p + 1] < v) bad = true;
        if (bad) L.ok = 0;
    }
    __syncthreads();
    if (tid == 0) *a.plan_ok = L.ok;                     // read by records_kernel
    if (!L.ok) {                                         // unusable shard table: plan nothing
        if (tid == 0) { set_status(a.status, DC_ERR_BAD_LAYOUT); *a.n_mb = 0; }
        return;
    }

    // ---- 1. permutation check (a repeat moves nothing), dense prefix of the slot lengths ----
    bool dup = false;
    for (int j = tid; j < N; j += PLANL_BLOCK) {
        const int32_t i = a.perm ? a.perm[j] : j;        // out-of-range entries were emptied by slots_kernel
        if (i >= 0 && i < N && ((atomicOr(&L.bits[i >> 5], 1u << (i & 31)) >> (i & 31)) & 1u)) {
            dup = true;
            a.slot_len[j] = 0;
        }
    }
    if (dup) set_status(a.status, DC_ERR_BAD_LAYOUT);
    __threadfence_block();
    __syncthreads();
    int64_t carry = 0;
    for (int base = 0; base < N; base += PLANL_BLOCK) {  // uniform
        const int j = base + tid;
        const int64_t len = j < N ? a.slot_len[j] : 0;
        int64_t total;
        const int64_t ex = block_excl_scan_add<int64_t>(len, L.tmp64, &total);
        if (j < N) a.gpre[j] = carry + ex;
        carry += total;
    }
    if (tid == 0) a.gpre[N] = carry;
    for (int i = tid; i < n_words; i += PLANL_BLOCK) L.bits[i] = 0;     // from here on: slot opens a micro-batch
    __threadfence_block();
    __syncthreads();

    // ---- 2. shard bases: exclusive scan of the loads rounded up to the alignment ----
    {
        const int64_t first = tid < P ? a.gpre[L.shard_off[tid]] : 0;
        const int64_t load = tid < P ? a.gpre[L.shard_off[tid + 1]] - first : 0;
        const int64_t padded = (load + a.align - 1) / a.align * a.align;
        int64_t end;
        const int64_t base = block_excl_scan_add<int64_t>(padded, L.tmp64, &end);
        if (tid < P) { L.shard_base[tid] = base; a.shard_tok_off[tid] = base; }
        if (tid == 0) {
            L.shard_base[P] = end;
            a.shard_tok_off[P] = end;
            a.dst_tok_off[N] = end;
            if (end > a.capacity) set_status(a.status, DC_ERR_OVERFLOW);
        }
    }

    // ---- 3. micro-batch starts: a group of lanes (few shards) or a lane (many) walks a shard ----
    if (P <= PLANL_WAVES * 4) {
        const int spw = P <= PLANL_WAVES ? 1 : (P <= 2 * PLANL_WAVES ? 2 : 4);     // shards per wave
        const int G = WAVE / spw, g = lane / G, gl = lane - g * G;
        const uint64_t group_mask = (G == WAVE ? ~0ull : (1ull << G) - 1ull);
        const int p = w * spw + g;
        if (p < P) {
            const int b = L.shard_off[p + 1];
            int j = L.shard_off[p];
            while (j < b) {                                  // uniform over the group
                if (gl == 0) atomicOr(&L.bits[j >> 5], 1u << (j & 31));
                const int64_t limit = a.gpre[j] + a.budget;
                int lo = j + 1, e = j + 1;                   // an over-budget slot still advances by one
                for (int win = 0;; ++win) {
                    const int c = lo + gl;
                    const bool fits = c <= b && a.gpre[min(c, b)] <= limit;
                    const int cnt = __popcll((__ballot(fits) >> (g * G)) & group_mask);
                    if (cnt > 0) e = lo + cnt - 1;
                    if (cnt < G || lo + G > b) break;
                    lo += G;
                    if (win == 1) {                          // every lane of the group reads the same words
                        int l = e, h = b;
                        while (l < h) {
                            const int mid = (l + h + 1) >> 1;
                            if (a.gpre[mid] <= limit) l = mid; else h = mid - 1;
                        }
                        e = l;
                        break;
                    }
                }
                j = e;
            }
        }
    } else if (tid < P) {
        const int b = L.shard_off[tid + 1];
        int j = L.shard_off[tid];
        while (j < b) {
            atomicOr(&L.bits[j >> 5], 1u << (j & 31));
            const int64_t limit = a.gpre[j] + a.budget;
            int lo = j + 1, hi = b;                          // largest e in [lo, hi] with gpre[e] <= limit, else lo
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (a.gpre[mid] <= limit) lo = mid; else hi = mid - 1;
            }
            j = lo;
        }
    }
    __syncthreads();

    // ---- 4. per word of 32 slots: starts before it and the last start before it; then the outputs ----
    int32_t M = 0, last_before = -1;
    for (int wb = 0; wb < n_words; wb += PLANL_BLOCK) {      // uniform
        const int wi = wb + tid;
        const uint32_t bits = wi < n_words ? L.bits[wi] : 0u;
        int32_t n_here, max_here;
        const int32_t before = block_excl_scan_add<int32_t>((int32_t)__popc(bits), L.tmp32, &n_here);
        const int32_t last = block_excl_scan_max_total(bits ? wi * 32 + 31 - __clz(bits) : -1, L.tmp32, &max_here);
        if (wi < n_words) { a.word_starts[wi] = M + before; a.word_last[wi] = max(last_before, last); }
        M += n_here;
        last_before = max(last_before, max_here);
    }
    if (tid == 0) a.word_starts[n_words] = M;
    __threadfence_block();
    __syncthreads();
    for (int j = tid; j < N; j += PLANL_BLOCK) {
        const uint32_t bits = L.bits[j >> 5];
        const uint32_t upto = bits & (0xFFFFFFFFu >> (31 - (j & 31)));           // starts at slots <= j of the word
        const int32_t m = a.word_starts[j >> 5] + (int32_t)__popc(upto) - 1;     // my micro-batch
        const int32_t cur_start = upto ? (j & ~31) + 31 - __clz(upto) : a.word_last[j >> 5];
        if ((bits >> (j & 31)) & 1u) a.mb_seq_off[m] = j;
        const int64_t g = a.gpre[j];
        int64_t d = g;
        if (a.align != 1) {                                  // uniform: shard of the slot, then its aligned base
            int lo = 0, hi = P - 1;                          // largest p with shard_off[p] <= j
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (L.shard_off[mid] <= j) lo = mid; else hi = mid - 1;
            }
            d = g + (L.shard_base[lo] - a.gpre[L.shard_off[lo]]);
        }
        a.dst_tok_off[j] = d;
        const int64_t gs = a.gpre[cur_start >= 0 ? cur_start : 0];
        a.cu_seqlens[j + m] = (int32_t)(g - gs);
        const bool closes = (j + 1 == N) || ((L.bits[(j + 1) >> 5] >> ((j + 1) & 31)) & 1u);
        if (closes) a.cu_seqlens[j + m + 1] = (int32_t)(a.gpre[j + 1] - gs);
    }
    for (int p = tid; p <= P; p += PLANL_BLOCK) {            // micro-batches before each shard's first slot
        const int js = L.shard_off[p];
        int32_t c = M;
        if (js < N) c = a.word_starts[js >> 5] + (int32_t)__popc(L.bits[js >> 5] & ((1u << (js & 31)) - 1u));
        a.shard_mb_off[p] = c;
    }
    if (tid == 0) { *a.n_mb = M; a.mb_seq_off[M] = N; }
}

hipError_t launch_plan_large(const PlanArgs& a, hipStream_t st) {
    if (a.n_seq > DC_MAX_SEQ_LARGE || !a.gpre || !a.word_starts || !a.word_last) return hipErrorInvalidValue;
    hipLaunchKernelGGL(plan_large_kernel, dim3(1), dim3(PLANL_BLOCK), 0, st, a);
    return hipGetLastError();
}

}  // namespace dc
