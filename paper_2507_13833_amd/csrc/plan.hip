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
#include "plan_device.h"

namespace dc {


// Per-slot source descriptors (one lane per slot, many workgroups; runs before plan_kernel on
// the same stream): the sequence behind each slot, its length and place in the rollout layout,
// validated; a slot that fails a check gets length 0 and moves nothing.  These are random
// gathers over seq_len / src_tok_off, which one workgroup alone could not keep in flight.
constexpr int SLOTS_BLOCK = 256;

// The sequence behind slot j with its place in the rollout layout, validated (what the gather may rely
// on): ln = tokens to move (0 if a check fails), so = element offset in rollout shard sh.  ln_in < 0: the
// length is taken from a.seq_len; else it is the slot's length as the caller has it already.  Sets the
// device status on a failed check (and on a sequence above the token budget, which is still laid out).
__device__ __forceinline__ void slot_source(const PlanArgs& a, const SourceDesc& sd, int j, int32_t ln_in,
                                            int32_t* ln_out, int64_t* so_out, int32_t* sh_out) {
    const int N = a.n_seq;
    const int32_t i = a.perm ? a.perm[j] : j;                                     // no permutation: slot j holds sequence j
    const bool placed = i >= 0 && i < N;
    int32_t ln = placed ? (ln_in < 0 ? a.seq_len[i] : ln_in) : 0;
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
    *ln_out = ln;
    *so_out = placed ? so : 0;
    *sh_out = sh;
}

__global__ __launch_bounds__(SLOTS_BLOCK) void slots_kernel(PlanArgs a, SourceDesc sd) {
    const int j = blockIdx.x * SLOTS_BLOCK + threadIdx.x;
    const int N = a.n_seq;
    if (a.own_shard_off && j <= sd.n_src) a.own_shard_off[j] = sd.seq_off[j];     // the plan keeps the rollout shards
    if (j >= N) return;
    int32_t ln, sh;
    int64_t so;
    slot_source(a, sd, j, -1, &ln, &so, &sh);
    a.slot_src_off[j] = so;
    a.slot_len[j] = ln;
    a.slot_shard[j] = sh;
}

__global__ __launch_bounds__(PLAN_BLOCK) void plan_kernel(PlanArgs a) {
    __shared__ PlanLds L;
    const int tid = threadIdx.x;
    const int N = a.n_seq;
    // the slots' sequences and lengths (validated by slots_kernel): asked for first, so that these loads are in
    // flight while the shard table is fetched and checked
    int32_t seq[PLAN_IPT], len[PLAN_IPT];
#pragma unroll
    for (int q = 0; q < PLAN_IPT; ++q) {
        const int j = q * PLAN_BLOCK + tid;
        seq[q] = j < N ? (a.perm ? a.perm[j] : j) : -1;
        len[q] = j < N ? a.slot_len[j] : 0;
    }
    plan_body(L, a, seq, len, true, 0);
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

// The first slot j of a token axis (starts[N + 1], the last entry its end) whose successor starts after `begin`, or N:
// what build_record's bisection finds, for the REC_BLOCK consecutive granules of a workgroup together (every thread of
// the workgroup must call it; begin must not decrease with the thread index).  A bisection of its own is 14 dependent
// reads of global memory per lane at 16 384 slots.  Here the workgroup reads REC_BLOCK evenly spaced starts at once,
// every lane finds its stretch between two of them in the LDS, the workgroup reads the stretches of all its lanes
// (one run of starts: the granules are neighbours) and every lane bisects its own stretch in the LDS: two reads of
// global memory in a row.  A run longer than REC_STAGE entries is bisected where it lies.
constexpr int REC_STAGE = 1024;
struct RecLds {
    int64_t sample[REC_BLOCK];
    int64_t stage[REC_STAGE];
    int32_t run_lo, run_hi;
};
__device__ __forceinline__ int first_slot_after(RecLds& L, int N, const int64_t* starts, int64_t begin) {
    const int tid = threadIdx.x;
    const int stride = (N + REC_BLOCK - 1) / REC_BLOCK;              // >= 1 (N > 0)
    L.sample[tid] = starts[min(tid * stride, N)];
    __syncthreads();
    // the last sample that does not lie after `begin` (sample 0 is starts[0] = 0 <= begin)
    int i = 0;
#pragma unroll
    for (int step = REC_BLOCK / 2; step >= 1; step >>= 1)
        if (L.sample[i + step] <= begin) i += step;
    // the answer lies in [lo, hi]: everything before sample i starts at or before `begin`; the slot before sample i + 1
    // has a successor behind `begin` (no sample i + 1: hi = N stands for "none")
    int lo = min(i * stride, N);
    int hi = i + 1 < REC_BLOCK ? min((i + 1) * stride, N) - 1 : N;
    hi = max(hi, lo);
    if (tid == 0) L.run_lo = lo;
    if (tid == REC_BLOCK - 1) L.run_hi = hi;
    __syncthreads();
    const int run_lo = L.run_lo, run_hi = L.run_hi;                   // the bisections read starts[run_lo + 1 .. run_hi]
    const bool staged = run_hi - run_lo + 1 <= REC_STAGE;             // (uniform)
    if (staged)
        for (int k = tid; k <= run_hi - run_lo; k += REC_BLOCK) L.stage[k] = starts[min(run_lo + k, N)];
    __syncthreads();
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        const int64_t next = staged ? L.stage[mid + 1 - run_lo] : starts[mid + 1];
        if (next > begin) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// Tables of granule g of a token axis holding N slots (starts[N+1], the last entry its end);
// usable = false leaves the granule empty.  desc(j, &ln, &so, &sh): the validated source of slot j.
// found >= 0: the first slot whose successor starts after the granule's first token (else it is looked for here).
template <typename Desc>
__device__ __forceinline__ void build_record(int N, bool usable, const int64_t* starts, Desc desc, int64_t g,
                                             int32_t* first_out, GranRec* rec_out, int found = -1) {
    const int64_t begin = g * GATHER_GRAN;
    int first = N;
    if (usable && N > 0) {
        // first j whose successor starts after `begin` ...
        int lo = 0, hi = N;
        if (found >= 0) lo = hi = found;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (starts[mid + 1] > begin) hi = mid; else lo = mid + 1;
        }
        // ... and if `begin` lies in the padding behind that slot (or the slot is empty), the next one
        while (lo < N) {
            int32_t ln, sh;
            int64_t so;
            desc(lo, &ln, &so, &sh);
            if (starts[lo] + ln > begin) break;
            ++lo;
        }
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
                int32_t ln, sh;
                int64_t so;
                desc(j, &ln, &so, &sh);
                rec.e[r].start = (int32_t)max(d, (int64_t)-REL_FAR);
                rec.e[r].lensh = ln | (sh << LENSH_SHIFT);
                rec.e[r].src_off = so;
            }
        }
    }
    *first_out = first;
    u32x4* out = reinterpret_cast<u32x4*>(rec_out);
    const u32x4* in = reinterpret_cast<const u32x4*>(&rec);
#pragma unroll
    for (int r = 0; r < REC_SLOTS; ++r) out[r] = in[r];
}

// The descriptors as slots_kernel left them in the workspace.
struct StoredDesc {
    const int64_t* slot_src_off;
    const int32_t* slot_len;
    const int32_t* slot_shard;
    __device__ __forceinline__ void operator()(int j, int32_t* ln, int64_t* so, int32_t* sh) const {
        *ln = slot_len[j]; *so = slot_src_off[j]; *sh = slot_shard[j];
    }
};

__global__ __launch_bounds__(REC_BLOCK) void records_kernel(RecArgs a) {
    __shared__ RecLds L;
    const int64_t g = (int64_t)blockIdx.x * REC_BLOCK + threadIdx.x;
    const bool usable = *a.plan_ok != 0;
    int found = -1;
    if (usable && a.n_seq > 0)                                   // (uniform) lanes behind the last granule look for its slot
        found = first_slot_after(L, a.n_seq, a.dst_tok_off, min(g, a.n_gran - 1) * GATHER_GRAN);
    if (g >= a.n_gran) return;
    build_record(a.n_seq, usable, a.dst_tok_off, StoredDesc{a.slot_src_off, a.slot_len, a.slot_shard}, g,
                 a.gran_first + g, a.gran_rec + g, found);
}

// The granule tables straight behind a launch that planned without slots_kernel (the plan as the balance
// workgroup's tail, which leaves the slots' lengths in the workspace): the first workgroups build the records,
// taking every slot's source through perm on the way; the others do slots_kernel's work for all slots (the
// gather reads those arrays only for tiles with many short sequences).  Both validate alike, so a record
// never depends on what the other workgroups have written yet.
__global__ __launch_bounds__(REC_BLOCK) void records_slots_kernel(RecArgs a, PlanArgs p, SourceDesc sd, uint32_t rec_blocks) {
    if (blockIdx.x < rec_blocks) {                               // (uniform)
        __shared__ RecLds L;
        const int64_t g = (int64_t)blockIdx.x * REC_BLOCK + threadIdx.x;
        const bool usable = *a.plan_ok != 0;
        int found = -1;
        if (usable && a.n_seq > 0)
            found = first_slot_after(L, a.n_seq, a.dst_tok_off, min(g, a.n_gran - 1) * GATHER_GRAN);
        if (g >= a.n_gran) return;
        build_record(a.n_seq, usable, a.dst_tok_off,
                     [&](int j, int32_t* ln, int64_t* so, int32_t* sh) { slot_source(p, sd, j, max(p.slot_len[j], 0), ln, so, sh); },
                     g, a.gran_first + g, a.gran_rec + g, found);
        return;
    }
    const int j = (int)(blockIdx.x - rec_blocks) * REC_BLOCK + (int)threadIdx.x;
    if (j >= p.n_seq) return;
    int32_t ln, sh;
    int64_t so;
    const int32_t had = p.slot_len[j];
    slot_source(p, sd, j, max(had, 0), &ln, &so, &sh);
    p.slot_src_off[j] = so;
    p.slot_shard[j] = sh;
    if (ln != had) p.slot_len[j] = ln;
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
    build_record(n, true, a.dst_tok_off + first_seq + s,
                 StoredDesc{a.slot_src_off + first_seq, a.slot_len + first_seq, a.slot_shard + first_seq},
                 g - gb, a.gran_first + g, a.gran_rec + g);
}

hipError_t launch_plan(const dc_params& prm, const SourceDesc& src, const int64_t* d_src_tok_off,
                       const int32_t* d_seq_len, const int32_t* d_perm, const int32_t* d_shard_seq_off,
                       int64_t dst_capacity, int64_t* d_dst_tok_off, int64_t* d_shard_tok_off,
                       int32_t* d_shard_mb_off, int32_t* d_mb_seq_off, int32_t* d_cu_seqlens,
                       int32_t* d_n_mb, const Workspace& ws, int32_t* d_status, hipStream_t st) {
    PlanArgs a = make_plan_args(prm, d_src_tok_off, d_seq_len, d_perm, d_shard_seq_off, dst_capacity, d_dst_tok_off,
                                d_shard_tok_off, d_shard_mb_off, d_mb_seq_off, d_cu_seqlens, d_n_mb, ws, d_status);
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

hipError_t launch_records_slots(const PlanArgs& p, const SourceDesc& src, const Workspace& ws, hipStream_t st) {
    RecArgs r;
    r.n_seq = p.n_seq; r.n_gran = ws.n_gran; r.dst_tok_off = p.dst_tok_off;
    r.slot_src_off = ws.slot_src_off; r.slot_len = ws.slot_len; r.slot_shard = ws.slot_shard;
    r.plan_ok = ws.plan_ok; r.gran_first = ws.gran_first; r.gran_rec = ws.gran_rec;
    const unsigned rec_blocks = (unsigned)((ws.n_gran + REC_BLOCK - 1) / REC_BLOCK);
    const unsigned slot_blocks = (unsigned)((p.n_seq + REC_BLOCK - 1) / REC_BLOCK);
    hipLaunchKernelGGL(records_slots_kernel, dim3(rec_blocks + slot_blocks), dim3(REC_BLOCK), 0, st, r, p, src, rec_blocks);
    return hipGetLastError();
}

PlanArgs make_plan_args(const dc_params& prm, const int64_t* d_src_tok_off, const int32_t* d_seq_len,
                        const int32_t* d_perm, const int32_t* d_shard_seq_off, int64_t dst_capacity,
                        int64_t* d_dst_tok_off, int64_t* d_shard_tok_off, int32_t* d_shard_mb_off,
                        int32_t* d_mb_seq_off, int32_t* d_cu_seqlens, int32_t* d_n_mb, const Workspace& ws,
                        int32_t* d_status) {
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
    return a;
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
