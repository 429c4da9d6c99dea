// Plan of the packed training layout: destination token offsets of every output
// slot, shard token offsets, next-fit micro-batches under the token budget and the
// per-micro-batch cu_seqlens, plus the gather's workspace (validated per-slot
// source descriptors and the first slot ending after every granule boundary of the
// destination token axis).
//
// O(N) integer work on at most DC_MAX_SEQ slots: latency-bound, so it runs as ONE
// workgroup of 1024 lanes with everything staged in LDS:
//   1. lane t owns slots [t*ipt, (t+1)*ipt): gathers len = seq_len[perm[j]],
//      validates, block-wide exclusive scan -> dense prefix gpre[0..N] (int64, LDS);
//   2. shard bases: serial over P <= 64 shards with the alignment round-up;
//   3. micro-batch starts: one lane per shard hops from start to start, each hop a
//      binary search for the last slot that still fits under the budget;
//   4. start flags -> micro-batch index by a block scan; outputs written in parallel.
#include "dc_device.h"
#include "dc_internal.h"

namespace dc {

constexpr int PLAN_BLOCK = 1024;
constexpr int PLAN_IPT = DC_MAX_SEQ / PLAN_BLOCK;        // slots per lane at the size limit

struct PlanArgs {
    int32_t n_seq, n_shards, align;
    int64_t budget, capacity, n_gran;
    const int64_t* src_tok_off;
    const int32_t* seq_len;
    const int32_t* perm;
    const int32_t* shard_seq_off;
    int64_t* dst_tok_off;
    int64_t* shard_tok_off;
    int32_t* shard_mb_off;
    int32_t* mb_seq_off;
    int32_t* cu_seqlens;
    int32_t* n_mb;
    int64_t* slot_src_off;
    int32_t* slot_len;
    int32_t* slot_shard;
    int32_t* gran_first;
    int32_t* status;
};

struct PlanLds {
    int64_t  gpre[DC_MAX_SEQ + 1];          // dense exclusive prefix of slot lengths
    uint32_t start_bits[DC_MAX_SEQ / 32];   // slot opens a micro-batch
    uint32_t seen_bits[DC_MAX_SEQ / 32];    // sequence already placed (perm must be a permutation)
    int64_t  shard_base[DC_MAX_SHARDS + 1]; // aligned token offset of each shard
    int32_t  shard_off[DC_MAX_SHARDS + 1];  // copy of shard_seq_off
    int32_t  lane_cnt[PLAN_BLOCK];          // exclusive count of starts before the lane's slots
    int64_t  tmp64[16];
    int32_t  tmp32[16];
    int32_t  ok;
};

__global__ __launch_bounds__(PLAN_BLOCK) void plan_kernel(PlanArgs a, SourceDesc sd) {
    __shared__ PlanLds L;
    const int tid = threadIdx.x;
    const int N = a.n_seq, P = a.n_shards;
    const int ipt = max(1, (N + PLAN_BLOCK - 1) / PLAN_BLOCK);   // <= PLAN_IPT
    const int j0 = tid * ipt;

    for (int i = tid; i < DC_MAX_SEQ / 32; i += PLAN_BLOCK) { L.start_bits[i] = 0; L.seen_bits[i] = 0; }
    // default: no slot ends after the granule boundary; step 4 overwrites the others
    for (int64_t t = tid; t < a.n_gran; t += PLAN_BLOCK) a.gran_first[t] = N;
    if (tid == 0) L.ok = 1;
    __syncthreads();
    if (tid <= P) {
        const int32_t v = a.shard_seq_off[tid];
        L.shard_off[tid] = v;
        bool bad = v < 0 || v > N || (tid == 0 && v != 0) || (tid == P && v != N);
        if (tid < P && a.shard_seq_off[tid + 1] < v) bad = true;
        if (bad) L.ok = 0;
    }
    __syncthreads();
    if (!L.ok) {                                         // unusable shard table: plan nothing
        if (tid == 0) { set_status(a.status, DC_ERR_BAD_LAYOUT); *a.n_mb = 0; }
        return;
    }

    // ---- 1. slot lengths, validation, dense prefix ----
    int32_t len[PLAN_IPT];
    int64_t mine = 0;
#pragma unroll
    for (int q = 0; q < PLAN_IPT; ++q) {
        const int j = j0 + q;
        len[q] = 0;
        if (q < ipt && j < N) {
            const int32_t i = a.perm[j];
            int32_t ln = 0, sh = 0;
            int64_t so = 0;
            if (i < 0 || i >= N) {
                set_status(a.status, DC_ERR_BAD_LAYOUT);
            } else if (atomicOr(&L.seen_bits[i >> 5], 1u << (i & 31)) & (1u << (i & 31))) {
                set_status(a.status, DC_ERR_BAD_LAYOUT);
            } else {
                ln = a.seq_len[i];
                so = a.src_tok_off[i];
                while (sh + 1 < sd.n_src && i >= sd.seq_off[sh + 1]) ++sh;
                if (ln <= 0 || ln > DC_MAX_SEQ_LEN) {
                    set_status(a.status, DC_ERR_ZERO_LENGTH_SEQ);
                    ln = 0;
                } else if (so < 0 || so + ln > sd.tokens[sh]) {
                    set_status(a.status, DC_ERR_BAD_LAYOUT);
                    ln = 0;
                } else if (ln > a.budget) {
                    set_status(a.status, DC_ERR_SEQ_EXCEEDS_BUDGET);   // still laid out, alone in its micro-batch
                }
            }
            len[q] = ln;
            a.slot_src_off[j] = so;
            a.slot_len[j] = ln;
            a.slot_shard[j] = sh;
            mine += ln;
        }
    }
    int64_t total;
    int64_t run = block_excl_scan_add<int64_t>(mine, L.tmp64, &total);
#pragma unroll
    for (int q = 0; q < PLAN_IPT; ++q) {
        const int j = j0 + q;
        if (q < ipt && j < N) { L.gpre[j] = run; run += len[q]; }
    }
    if (tid == 0) L.gpre[N] = total;
    __syncthreads();

    // ---- 2. shard bases (alignment round-up is a serial dependency over <= 64 shards) ----
    if (tid == 0) {
        int64_t pos = 0;
        for (int p = 0; p < P; ++p) {
            L.shard_base[p] = pos;
            a.shard_tok_off[p] = pos;
            pos += L.gpre[L.shard_off[p + 1]] - L.gpre[L.shard_off[p]];
            pos = (pos + a.align - 1) / a.align * a.align;
        }
        L.shard_base[P] = pos;
        a.shard_tok_off[P] = pos;
        a.dst_tok_off[N] = pos;
        if (pos > a.capacity) set_status(a.status, DC_ERR_OVERFLOW);
    }

    // ---- 3. micro-batch starts: lane p walks shard p ----
    if (tid < P) {
        const int b = L.shard_off[tid + 1];
        int j = L.shard_off[tid];
        while (j < b) {
            atomicOr(&L.start_bits[j >> 5], 1u << (j & 31));
            const int64_t limit = L.gpre[j] + a.budget;
            int lo = j + 1, hi = b;                      // largest e in [j+1, b] with gpre[e] <= limit
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (L.gpre[mid] <= limit) lo = mid; else hi = mid - 1;
            }
            j = lo;                                      // an over-budget slot still advances by one
        }
    }
    __syncthreads();

    // ---- 4. micro-batch index per slot, outputs ----
    int32_t n_start = 0, last_start = -1;
#pragma unroll
    for (int q = 0; q < PLAN_IPT; ++q) {
        const int j = j0 + q;
        if (q < ipt && j < N && ((L.start_bits[j >> 5] >> (j & 31)) & 1u)) { ++n_start; last_start = j; }
    }
    int32_t M;
    int32_t m_before = block_excl_scan_add<int32_t>(n_start, L.tmp32, &M);
    int32_t cur_start = block_excl_scan_max(last_start, L.tmp32);   // start slot of the batch open at j0
    L.lane_cnt[tid] = m_before;
    __syncthreads();

    int p = 0;                                           // shard of slot j0
    if (j0 < N) while (p + 1 < P && j0 >= L.shard_off[p + 1]) ++p;
    int32_t m = m_before - 1;                            // index of the micro-batch open at j0
#pragma unroll
    for (int q = 0; q < PLAN_IPT; ++q) {
        const int j = j0 + q;
        if (q < ipt && j < N) {
            while (p + 1 < P && j >= L.shard_off[p + 1]) ++p;
            const bool opens = (L.start_bits[j >> 5] >> (j & 31)) & 1u;
            if (opens) { ++m; cur_start = j; a.mb_seq_off[m] = j; }
            const int64_t g = L.gpre[j];
            const int64_t d = L.shard_base[p] + (g - L.gpre[L.shard_off[p]]);
            a.dst_tok_off[j] = d;
            const int64_t gs = L.gpre[cur_start];
            a.cu_seqlens[j + m] = (int32_t)(g - gs);
            const bool closes = (j + 1 == N) || ((L.start_bits[(j + 1) >> 5] >> ((j + 1) & 31)) & 1u);
            if (closes) a.cu_seqlens[j + m + 1] = (int32_t)(L.gpre[j + 1] - gs);

            // granule boundaries b with end(j-1) <= b < end(j): j is the first slot ending after b
            const int64_t ln = L.gpre[j + 1] - g;
            if (ln > 0) {
                int64_t prev_end = 0;
                if (j > 0) {
                    int pp = p;                          // shard of slot j-1
                    while (pp > 0 && j - 1 < L.shard_off[pp]) --pp;
                    prev_end = L.shard_base[pp] + (g - L.gpre[L.shard_off[pp]]);
                }
                int64_t t = (prev_end + GATHER_GRAN - 1) / GATHER_GRAN;
                for (; t < a.n_gran && t * GATHER_GRAN < d + ln; ++t) a.gran_first[t] = j;
            }
        }
    }
    if (tid <= P) {                                      // micro-batches before each shard's first slot
        const int js = L.shard_off[tid];
        int32_t c;
        if (js >= N) {
            c = M;
        } else {
            const int owner = js / ipt;
            c = L.lane_cnt[owner];
            for (int j = owner * ipt; j < js; ++j) c += (L.start_bits[j >> 5] >> (j & 31)) & 1u;
        }
        a.shard_mb_off[tid] = c;
    }
    if (tid == 0) { *a.n_mb = M; a.mb_seq_off[M] = N; }
}

// Inline slot descriptors per granule (one lane per granule): the first REC_SLOTS slots
// from gran_first[g] on, as long as they start before the granule's end.  Runs after
// plan_kernel on the same stream.
constexpr int REC_BLOCK = 256;

struct RecArgs {
    int32_t        n_seq;
    int64_t        n_gran;
    const int64_t* dst_tok_off;
    const int64_t* slot_src_off;
    const int32_t* slot_len;
    const int32_t* slot_shard;
    const int32_t* gran_first;
    GranRec*       gran_rec;
};

__global__ __launch_bounds__(REC_BLOCK) void records_kernel(RecArgs a) {
    const int64_t g = (int64_t)blockIdx.x * REC_BLOCK + threadIdx.x;
    if (g >= a.n_gran) return;
    const int N = a.n_seq;
    const int first = a.gran_first[g];
    const int next = g + 1 < a.n_gran ? a.gran_first[g + 1] : N;
    const int last = min(next, N - 1);
    const int64_t begin = g * GATHER_GRAN;
    GranRec rec;
#pragma unroll
    for (int r = 0; r < REC_SLOTS; ++r) {
        rec.e[r].start = REL_FAR; rec.e[r].lensh = 0; rec.e[r].src_off = 0;
        const int j = first + r;
        if (first >= 0 && first < N && j <= last) {
            const int64_t d = a.dst_tok_off[j] - begin;
            if (d < GATHER_GRAN) {
                rec.e[r].start = (int32_t)max(d, (int64_t)-REL_FAR);
                rec.e[r].lensh = a.slot_len[j] | (a.slot_shard[j] << LENSH_SHIFT);
                rec.e[r].src_off = a.slot_src_off[j];
            }
        }
    }
    u32x4* out = reinterpret_cast<u32x4*>(&a.gran_rec[g]);
    const u32x4* in = reinterpret_cast<const u32x4*>(&rec);
#pragma unroll
    for (int r = 0; r < REC_SLOTS; ++r) out[r] = in[r];
}

hipError_t launch_plan(const dc_params& prm, const SourceDesc& src, const int64_t* d_src_tok_off,
                       const int32_t* d_seq_len, const int32_t* d_perm, const int32_t* d_shard_seq_off,
                       int64_t dst_capacity, int64_t* d_dst_tok_off, int64_t* d_shard_tok_off,
                       int32_t* d_shard_mb_off, int32_t* d_mb_seq_off, int32_t* d_cu_seqlens,
                       int32_t* d_n_mb, const Workspace& ws, int32_t* d_status, hipStream_t st) {
    PlanArgs a;
    a.n_seq = prm.n_seq; a.n_shards = prm.n_shards; a.align = prm.align_tokens;
    a.budget = prm.token_budget; a.capacity = dst_capacity; a.n_gran = ws.n_gran;
    a.src_tok_off = d_src_tok_off; a.seq_len = d_seq_len; a.perm = d_perm; a.shard_seq_off = d_shard_seq_off;
    a.dst_tok_off = d_dst_tok_off; a.shard_tok_off = d_shard_tok_off; a.shard_mb_off = d_shard_mb_off;
    a.mb_seq_off = d_mb_seq_off; a.cu_seqlens = d_cu_seqlens; a.n_mb = d_n_mb;
    a.slot_src_off = ws.slot_src_off; a.slot_len = ws.slot_len; a.slot_shard = ws.slot_shard;
    a.gran_first = ws.gran_first; a.status = d_status;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(PLAN_BLOCK), 0, st, a, src);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    RecArgs r;
    r.n_seq = prm.n_seq; r.n_gran = ws.n_gran; r.dst_tok_off = d_dst_tok_off;
    r.slot_src_off = ws.slot_src_off; r.slot_len = ws.slot_len; r.slot_shard = ws.slot_shard;
    r.gran_first = ws.gran_first; r.gran_rec = ws.gran_rec;
    hipLaunchKernelGGL(records_kernel, dim3((unsigned)((ws.n_gran + REC_BLOCK - 1) / REC_BLOCK)), dim3(REC_BLOCK), 0, st, r);
    return hipGetLastError();
}

}  // namespace dc
