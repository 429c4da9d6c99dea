// Plan of the packed training layout: destination token offsets of every output
// slot, shard token offsets, next-fit micro-batches under the token budget and the
// per-micro-batch cu_seqlens, plus the gather's workspace (validated per-slot
// source descriptors and, per 1024-token granule of the destination, the first slot
// reaching into it and the record of the slots that do).
//
// O(N) integer work on at most DC_MAX_SEQ slots: latency-bound, so the plan proper runs as
// ONE workgroup of 1024 lanes with everything staged in LDS.  Lane t handles slots t,
// t + 1024, ... (every global access is coalesced):
//   0. (slots_kernel, many workgroups) len = seq_len[perm[j]] and the rollout offset of every
//      slot, validated: random gathers, which need more loads in flight than one CU has;
//   1. slot lengths, check that perm is a permutation; wave scans + one scan of the 256 wave
//      totals -> dense prefix gpre[0..N] (int64, LDS);
//   2. shard bases: exclusive scan of the shard loads, each rounded up to the alignment (a base is
//      always a multiple of it, so rounding the running sum equals summing the rounded loads);
//   3. micro-batch starts: one lane per shard hops from start to start, each hop a
//      bisection for the last slot that still fits under the budget -> start bits;
//   4. per 32 slots: starts before the word and the last start before it (two scans over
//      512 words); then every slot reads its micro-batch index and start from those and
//      writes its outputs.
#include "dc_device.h"
#include "dc_internal.h"
#include "dc_lanes.h"

namespace dc {

constexpr int PLAN_BLOCK = 1024;
constexpr int PLAN_WAVES = PLAN_BLOCK / WAVE;
constexpr int PLAN_IPT = DC_MAX_SEQ / PLAN_BLOCK;        // slots per lane at the size limit
constexpr int PLAN_WORDS = DC_MAX_SEQ / 32;


struct PlanLds {
    int64_t  gpre[DC_MAX_SEQ + 1];          // dense exclusive prefix of slot lengths
    uint32_t start_bits[PLAN_WORDS];        // slot opens a micro-batch
    uint32_t seen_bits[PLAN_WORDS];         // sequence already placed (perm must be a permutation)
    int32_t  word_starts[PLAN_WORDS + 1];   // starts in the words before this one
    int32_t  word_last[PLAN_WORDS];         // last start in the words before this one, or -1
    int64_t  wave_pref[PLAN_IPT * PLAN_WAVES];  // tokens before the 64 slots a wave handles in one step
    int64_t  shard_base[DC_MAX_SHARDS + 1]; // aligned token offset of each shard
    int32_t  shard_off[DC_MAX_SHARDS + 1];  // copy of shard_seq_off
    int64_t  tmp64[16];
    int32_t  tmp32[16];
    int32_t  ok;
};

// Per-slot source descriptors (one lane per slot, many workgroups; runs before plan_kernel on
// the same stream): the sequence behind each slot, its length and place in the rollout layout,
// validated; a slot that fails a check gets length 0 and moves nothing.  These are random
// gathers over seq_len / src_tok_off, which one workgroup alone could not keep in flight.
constexpr int SLOTS_BLOCK = 256;

__global__ __launch_bounds__(SLOTS_BLOCK) void slots_kernel(PlanArgs a, SourceDesc sd) {
    const int j = blockIdx.x * SLOTS_BLOCK + threadIdx.x;
    const int N = a.n_seq;
    if (a.own_shard_off && j <= sd.n_src) a.own_shard_off[j] = sd.seq_off[j];     // the plan keeps the rollout shards
    if (j >= N) return;
    const int32_t i = a.perm ? a.perm[j] : j;                                     // no permutation: slot j holds sequence j
    const bool placed = i >= 0 && i < N;
    int32_t ln = placed ? a.seq_len[i] : 0;
    const int64_t so = placed ? a.src_tok_off[i] : 0;
    int32_t sh = 0;                                      // rollout shard (seq_off[s] = N from s = n_src on)
    if (sd.n_src > 1 && placed) {
#pragma unroll
        for (int s = 1; s < DC_MAX_SRC_SHARDS; ++s) sh += i >= sd.seq_off[s] ? 1 : 0;
    }
    int64_t tokens = sd.tokens[0];
#pragma unroll
    for (int s = 1; s < DC_MAX_SRC_SHARDS; ++s) tokens = sh == s ? sd.tokens[s] : tokens;
    const bool bad_len = placed && (ln <= 0 || ln > DC_MAX_SEQ_LEN);
    const bool bad_off = placed && !bad_len && (so < 0 || so + ln > tokens);
    const bool over = placed && !bad_len && !bad_off && ln > a.budget;   // still laid out, alone in its micro-batch
    const int32_t e = !placed ? DC_ERR_BAD_LAYOUT
                      : bad_len ? DC_ERR_ZERO_LENGTH_SEQ
                      : bad_off ? DC_ERR_BAD_LAYOUT
                      : over ? DC_ERR_SEQ_EXCEEDS_BUDGET : 0;
    if (e != 0) set_status(a.status, e);
    if (!placed || bad_len || bad_off) ln = 0;
    a.slot_src_off[j] = placed ? so : 0;
    a.slot_len[j] = ln;
    a.slot_shard[j] = sh;
}

__device__ __forceinline__ bool start_bit(const PlanLds& L, int j) { return (L.start_bits[j >> 5] >> (j & 31)) & 1u; }

__global__ __launch_bounds__(PLAN_BLOCK) void plan_kernel(PlanArgs a) {
    __shared__ PlanLds L;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    const int N = a.n_seq, P = a.n_shards;
    const int nb = (N + PLAN_BLOCK - 1) / PLAN_BLOCK;    // steps of 1024 slots, <= PLAN_IPT

    // the slots' sequences and lengths (validated by slots_kernel): asked for first, so that these loads are in
    // flight while the shard table is fetched and checked
    int32_t seq[PLAN_IPT], len[PLAN_IPT];
#pragma unroll
    for (int q = 0; q < PLAN_IPT; ++q) {
        const int j = q * PLAN_BLOCK + tid;
        seq[q] = j < N ? (a.perm ? a.perm[j] : j) : -1;
        len[q] = j < N ? a.slot_len[j] : 0;
    }

    for (int i = tid; i < PLAN_WORDS; i += PLAN_BLOCK) { L.start_bits[i] = 0; L.seen_bits[i] = 0; }
    if (tid == 0) L.ok = 1;
    __syncthreads();
    for (int p = tid; p <= P; p += PLAN_BLOCK) {         // P + 1 entries, P up to the block size
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

    // ---- 1. permutation check, dense prefix of the slot lengths ----
    uint32_t dup = 0;                                    // bit q: perm repeats an earlier entry at my slot of step q
#pragma unroll
    for (int q = 0; q < PLAN_IPT; ++q) {
        const int32_t i = seq[q];                        // -1 beyond N; out-of-range entries were emptied by slots_kernel
        if (i >= 0 && i < N) dup |= ((atomicOr(&L.seen_bits[i >> 5], 1u << (i & 31)) >> (i & 31)) & 1u) << q;
    }
    if (__ballot(dup != 0) != 0ull) {                    // uniform, rare: perm is not a permutation; a repeat moves nothing
        if (dup != 0) set_status(a.status, DC_ERR_BAD_LAYOUT);
#pragma unroll
        for (int q = 0; q < PLAN_IPT; ++q)
            if ((dup >> q) & 1u) { len[q] = 0; a.slot_len[q * PLAN_BLOCK + tid] = 0; }
    }
    // dense prefix: inclusive scan inside each wave step (a wave's 64 slots hold < 2^31 tokens) ...
    int32_t inc[PLAN_IPT];
#pragma unroll
    for (int q = 0; q < PLAN_IPT; ++q) {
        inc[q] = (int32_t)wave_incl_scan_add_u32((uint32_t)len[q]);
        if (lane == WAVE - 1) L.wave_pref[q * PLAN_WAVES + w] = inc[q];
    }
    __syncthreads();
    // ... an exclusive scan of the 256 step totals in slot order (step q, wave w) ...
    {
        const int64_t v = tid < PLAN_IPT * PLAN_WAVES ? L.wave_pref[tid] : 0;
        int64_t total;
        const int64_t ex = block_excl_scan_add<int64_t>(v, L.tmp64, &total);
        if (tid < PLAN_IPT * PLAN_WAVES) L.wave_pref[tid] = ex;
        if (tid == 0) L.gpre[N] = total;
    }
    __syncthreads();
    // ... and their sum
#pragma unroll
    for (int q = 0; q < PLAN_IPT; ++q) {
        const int j = q * PLAN_BLOCK + tid;
        if (j < N) L.gpre[j] = L.wave_pref[q * PLAN_WAVES + w] + (inc[q] - len[q]);
    }
    __syncthreads();

    // ---- 2. shard bases: lane p takes shard p; exclusive scan of the loads rounded up to the alignment ----
    {
        const int64_t first = tid < P ? L.gpre[L.shard_off[tid]] : 0;
        const int64_t load = tid < P ? L.gpre[L.shard_off[tid + 1]] - first : 0;
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

    // ---- 3. micro-batch starts ----
    // Many shards: lane p walks shard p.
    // Each hop looks for the last slot that still fits under the budget.  Slots of a shard come in
    // descending length, so a micro-batch holds about as many slots as the one before it: the
    // search gallops outwards from that guess and bisects what is left (a few probes of the prefix
    // instead of log2 N per hop; the hops of a shard are one dependent chain).
    if (P <= PLAN_WAVES * 4) {
        // Few shards: a group of 64, 32 or 16 LANES walks a shard (every wave takes 1, 2 or 4 shards).  A
        // hop probes the slots behind the micro-batch's start G at a time, one per lane: the prefix sums
        // do not decrease, so the lanes that still fit are a prefix of the group and a ballot counts them -
        // one LDS round trip per window where the dependent probes of a search take six to eight.  A
        // micro-batch of more than two windows finishes with a bisection.
        const int spw = P <= PLAN_WAVES ? 1 : (P <= 2 * PLAN_WAVES ? 2 : 4);     // shards per wave
        const int G = WAVE / spw, g = lane / G, gl = lane - g * G;
        const uint64_t group_mask = (G == WAVE ? ~0ull : (1ull << G) - 1ull);
        const int p = w * spw + g;
        if (p < P) {
            const int b = L.shard_off[p + 1];
            int j = L.shard_off[p];
            while (j < b) {                                  // uniform over the group
                if (gl == 0) atomicOr(&L.start_bits[j >> 5], 1u << (j & 31));
                const int64_t limit = L.gpre[j] + a.budget;
                int lo = j + 1, e = j + 1;                   // an over-budget slot still advances by one
                for (int win = 0;; ++win) {
                    const int c = lo + gl;
                    const bool fits = c <= b && L.gpre[min(c, b)] <= limit;
                    const int cnt = __popcll((__ballot(fits) >> (g * G)) & group_mask);
                    if (cnt > 0) e = lo + cnt - 1;
                    if (cnt < G || lo + G > b) break;
                    lo += G;
                    if (win == 1) {                          // every lane of the group reads the same words
                        int l = e, h = b;
                        while (l < h) {
                            const int mid = (l + h + 1) >> 1;
                            if (L.gpre[mid] <= limit) l = mid; else h = mid - 1;
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
        int sz = 1;                                      // slots in the previous micro-batch
        while (j < b) {
            atomicOr(&L.start_bits[j >> 5], 1u << (j & 31));
            const int64_t limit = L.gpre[j] + a.budget;
            int lo = j + 1, hi = b;                      // largest e in [lo, hi] with gpre[e] <= limit; gpre[lo] may
                                                         // exceed it: an over-budget slot still advances by one
            int g = min(j + sz, b);
            if (g > lo) {
                if (L.gpre[g] <= limit) {
                    lo = g;
                    for (int w = 1; lo < hi; w <<= 1) {  // gallop up
                        g = min(lo + w, hi);
                        if (L.gpre[g] <= limit) lo = g; else { hi = g - 1; break; }
                    }
                } else {
                    hi = g - 1;
                    for (int w = 1; lo < hi; w <<= 1) {  // gallop down
                        g = max(hi + 1 - w, lo);
                        if (g == lo) break;
                        if (L.gpre[g] <= limit) { lo = g; break; }
                        hi = g - 1;
                    }
                }
            }
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (L.gpre[mid] <= limit) lo = mid; else hi = mid - 1;
            }
            sz = lo - j;
            j = lo;
        }
    }
    __syncthreads();

    // ---- 4. micro-batch index per slot, outputs ----
    // per word of 32 slots: starts in the words before it, and the last start before it
    int32_t M;
    {
        const uint32_t bits = tid < PLAN_WORDS ? L.start_bits[tid] : 0u;
        const int32_t before = block_excl_scan_add<int32_t>((int32_t)__popc(bits), L.tmp32, &M);
        const int32_t last = block_excl_scan_max(bits ? tid * 32 + 31 - __clz(bits) : -1, L.tmp32);
        if (tid < PLAN_WORDS) { L.word_starts[tid] = before; L.word_last[tid] = last; }
        if (tid == 0) L.word_starts[PLAN_WORDS] = M;
    }
    __syncthreads();
#pragma unroll 2
    for (int q = 0; q < nb; ++q) {
        const int j = q * PLAN_BLOCK + tid;
        if (j < N) {
            const uint32_t bits = L.start_bits[j >> 5];
            const uint32_t upto = bits & (0xFFFFFFFFu >> (31 - (j & 31)));           // starts at slots <= j of the word
            const int32_t m = L.word_starts[j >> 5] + (int32_t)__popc(upto) - 1;     // my micro-batch
            const int32_t cur_start = upto ? (j & ~31) + 31 - __clz(upto) : L.word_last[j >> 5];
            if ((bits >> (j & 31)) & 1u) a.mb_seq_off[m] = j;
            const int64_t g = L.gpre[j];
            int64_t d = g;
            if (a.align != 1) {                          // uniform: shard of the slot, then its aligned base
                int lo = 0, hi = P - 1;                  // largest p with shard_off[p] <= j
                while (lo < hi) {
                    const int mid = (lo + hi + 1) >> 1;
                    if (L.shard_off[mid] <= j) lo = mid; else hi = mid - 1;
                }
                d = g + (L.shard_base[lo] - L.gpre[L.shard_off[lo]]);
            }
            a.dst_tok_off[j] = d;
            const int64_t gs = L.gpre[cur_start >= 0 ? cur_start : 0];
            a.cu_seqlens[j + m] = (int32_t)(g - gs);
            const bool closes = (j + 1 == N) || start_bit(L, j + 1);
            if (closes) a.cu_seqlens[j + m + 1] = (int32_t)(L.gpre[j + 1] - gs);
        }
    }
    for (int p = tid; p <= P; p += PLAN_BLOCK) {         // micro-batches before each shard's first slot
        const int js = L.shard_off[p];
        int32_t c = M;
        if (js < N) c = L.word_starts[js >> 5] + (int32_t)__popc(L.start_bits[js >> 5] & ((1u << (js & 31)) - 1u));
        a.shard_mb_off[p] = c;
    }
    if (tid == 0) { *a.n_mb = M; a.mb_seq_off[M] = N; }
}

// Per-granule tables for the gather (one lane per granule, many workgroups; runs after
// plan_kernel on the same stream): F[g] = first slot that ends after the granule's first
// token, found by bisection over the slot starts, and the record of the first REC_SLOTS
// slots from F[g] on that start before the granule's end.
constexpr int REC_BLOCK = 256;

struct RecArgs {
    int32_t        n_seq;
    int64_t        n_gran;
    const int64_t* dst_tok_off;      // [N+1]
    const int64_t* slot_src_off;
    const int32_t* slot_len;
    const int32_t* slot_shard;
    const int32_t* plan_ok;
    int32_t*       gran_first;
    GranRec*       gran_rec;
};

// Tables of granule g of a token axis holding N slots (starts[N+1], the last entry its end);
// usable = false leaves the granule empty.
__device__ __forceinline__ void build_record(int N, bool usable, const int64_t* starts, const int64_t* slot_src_off,
                                             const int32_t* slot_len, const int32_t* slot_shard, int64_t g,
                                             int32_t* first_out, GranRec* rec_out) {
    const int64_t begin = g * GATHER_GRAN;
    int first = N;
    if (usable && N > 0) {
        // first j whose successor starts after `begin` ...
        int lo = 0, hi = N;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (starts[mid + 1] > begin) hi = mid; else lo = mid + 1;
        }
        // ... and if `begin` lies in the padding behind that slot (or the slot is empty), the next one
        while (lo < N && starts[lo] + slot_len[lo] <= begin) ++lo;
        first = lo;
    }
    GranRec rec;
#pragma unroll
    for (int r = 0; r < REC_SLOTS; ++r) {
        rec.e[r].start = REL_FAR; rec.e[r].lensh = 0; rec.e[r].src_off = 0;
        const int j = first + r;
        if (j < N) {
            const int64_t d = starts[j] - begin;
            if (d < GATHER_GRAN) {
                rec.e[r].start = (int32_t)max(d, (int64_t)-REL_FAR);
                rec.e[r].lensh = slot_len[j] | (slot_shard[j] << LENSH_SHIFT);
                rec.e[r].src_off = slot_src_off[j];
            }
        }
    }
    *first_out = first;
    u32x4* out = reinterpret_cast<u32x4*>(rec_out);
    const u32x4* in = reinterpret_cast<const u32x4*>(&rec);
#pragma unroll
    for (int r = 0; r < REC_SLOTS; ++r) out[r] = in[r];
}

__global__ __launch_bounds__(REC_BLOCK) void records_kernel(RecArgs a) {
    const int64_t g = (int64_t)blockIdx.x * REC_BLOCK + threadIdx.x;
    if (g >= a.n_gran) return;
    build_record(a.n_seq, *a.plan_ok != 0, a.dst_tok_off, a.slot_src_off, a.slot_len, a.slot_shard, g,
                 a.gran_first + g, a.gran_rec + g);
}

// The same for the reverse path: the granule tables of every rollout buffer, one behind the
// other; a.dst_tok_off holds the slot starts of segment s from index first_seq[s] + s on.
__global__ __launch_bounds__(REC_BLOCK) void records_back_kernel(RecArgs a, BackSegs bs) {
    const int64_t g = (int64_t)blockIdx.x * REC_BLOCK + threadIdx.x;
    if (g >= a.n_gran) return;
    int s = 0;
#pragma unroll
    for (int q = 1; q < DC_MAX_SRC_SHARDS; ++q) s += (q < bs.n_seg && g >= bs.gran_base[q]) ? 1 : 0;
    int32_t first_seq = bs.first_seq[0], n = bs.n_seq[0];
    int64_t gb = bs.gran_base[0];
#pragma unroll
    for (int q = 1; q < DC_MAX_SRC_SHARDS; ++q)
        if (s == q) { first_seq = bs.first_seq[q]; n = bs.n_seq[q]; gb = bs.gran_base[q]; }
    build_record(n, true, a.dst_tok_off + first_seq + s, a.slot_src_off + first_seq, a.slot_len + first_seq,
                 a.slot_shard + first_seq, g - gb, a.gran_first + g, a.gran_rec + g);
}

hipError_t launch_plan(const dc_params& prm, const SourceDesc& src, const int64_t* d_src_tok_off,
                       const int32_t* d_seq_len, const int32_t* d_perm, const int32_t* d_shard_seq_off,
                       int64_t dst_capacity, int64_t* d_dst_tok_off, int64_t* d_shard_tok_off,
                       int32_t* d_shard_mb_off, int32_t* d_mb_seq_off, int32_t* d_cu_seqlens,
                       int32_t* d_n_mb, const Workspace& ws, int32_t* d_status, hipStream_t st) {
    PlanArgs a;
    a.n_seq = prm.n_seq; a.n_shards = prm.n_shards; a.align = prm.align_tokens;
    a.budget = prm.token_budget; a.capacity = dst_capacity;
    a.src_tok_off = d_src_tok_off; a.seq_len = d_seq_len; a.perm = d_perm; a.shard_seq_off = d_shard_seq_off;
    a.dst_tok_off = d_dst_tok_off; a.shard_tok_off = d_shard_tok_off; a.shard_mb_off = d_shard_mb_off;
    a.mb_seq_off = d_mb_seq_off; a.cu_seqlens = d_cu_seqlens; a.n_mb = d_n_mb;
    a.slot_src_off = ws.slot_src_off; a.slot_len = ws.slot_len; a.slot_shard = ws.slot_shard;
    a.plan_ok = ws.plan_ok; a.status = d_status;
    a.gpre = ws.gpre; a.word_starts = ws.word_starts; a.word_last = ws.word_last;
    a.own_shard_off = nullptr;
    if (!d_shard_seq_off) { a.own_shard_off = ws.own_shard_off; a.shard_seq_off = ws.own_shard_off; }
    if (prm.n_seq > 0 || a.own_shard_off) {
        hipLaunchKernelGGL(slots_kernel, dim3((unsigned)max(1, (prm.n_seq + SLOTS_BLOCK - 1) / SLOTS_BLOCK)),
                           dim3(SLOTS_BLOCK), 0, st, a, src);
        hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
    }
    hipError_t e;
    if (prm.n_seq > DC_MAX_SEQ) {
        if (!ws.gpre) return hipErrorInvalidValue;
        e = launch_plan_large(a, st);
    } else {
        hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(PLAN_BLOCK), 0, st, a);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    return launch_records(prm.n_seq, d_dst_tok_off, ws, st);
}

hipError_t launch_records(int32_t n_seq, const int64_t* d_dst_tok_off, const Workspace& ws, hipStream_t st) {
    RecArgs r;
    r.n_seq = n_seq; r.n_gran = ws.n_gran; r.dst_tok_off = d_dst_tok_off;
    r.slot_src_off = ws.slot_src_off; r.slot_len = ws.slot_len; r.slot_shard = ws.slot_shard;
    r.plan_ok = ws.plan_ok; r.gran_first = ws.gran_first; r.gran_rec = ws.gran_rec;
    hipLaunchKernelGGL(records_kernel, dim3((unsigned)((ws.n_gran + REC_BLOCK - 1) / REC_BLOCK)), dim3(REC_BLOCK), 0, st, r);
    return hipGetLastError();
}

hipError_t launch_records_back(const BackSegs& bs, const ScatterWorkspace& ws, hipStream_t st) {
    RecArgs r;
    r.n_seq = 0; r.n_gran = ws.n_gran_all; r.dst_tok_off = ws.r_dst_off;
    r.slot_src_off = ws.r_src_off; r.slot_len = ws.r_len; r.slot_shard = ws.r_shard;
    r.plan_ok = nullptr; r.gran_first = ws.gran_first; r.gran_rec = ws.gran_rec;
    if (ws.n_gran_all <= 0) return hipSuccess;
    hipLaunchKernelGGL(records_back_kernel, dim3((unsigned)((ws.n_gran_all + REC_BLOCK - 1) / REC_BLOCK)), dim3(REC_BLOCK),
                       0, st, r, bs);
    return hipGetLastError();
}

}  // namespace dc
