// The plan proper (dense prefix of the slot lengths, shard bases, next-fit micro-batches, per-slot outputs)
// as device code of one workgroup of PLAN_BLOCK lanes, shared by plan_kernel (a launch of its own behind
// slots_kernel) and by the launch that runs it as the tail of the balance workgroup.
#pragma once
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


// The caller holds, per lane, the sequence and the (validated) length of slots tid, tid + PLAN_BLOCK, ...
// (seq = -1, len = 0 beyond N).  check_perm: seq comes from a caller's permutation and must be checked;
// fixed_c > 0: shard p owns slots [p * fixed_c, (p + 1) * fixed_c) and a.shard_seq_off is not read.
// Every lane of the workgroup must call it (barriers inside).
__device__ __forceinline__ void plan_body(PlanLds& L, const PlanArgs& a, int32_t (&seq)[PLAN_IPT], int32_t (&len)[PLAN_IPT],
                                          bool check_perm, int fixed_c) {
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    const int N = a.n_seq, P = a.n_shards;
    const int nb = (N + PLAN_BLOCK - 1) / PLAN_BLOCK;    // steps of 1024 slots, <= PLAN_IPT

    for (int i = tid; i < PLAN_WORDS; i += PLAN_BLOCK) { L.start_bits[i] = 0; L.seen_bits[i] = 0; }
    if (tid == 0) L.ok = 1;
    __syncthreads();
    for (int p = tid; p <= P; p += PLAN_BLOCK) {         // P + 1 entries, P up to the block size
        if (fixed_c > 0) { L.shard_off[p] = p * fixed_c; continue; }        // (uniform) N == P * fixed_c: nothing to check
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
    if (check_perm) {                                    // (uniform)
#pragma unroll
        for (int q = 0; q < PLAN_IPT; ++q) {
            const int32_t i = seq[q];                    // -1 beyond N; out-of-range entries were emptied by slots_kernel
            if (i >= 0 && i < N) dup |= ((atomicOr(&L.seen_bits[i >> 5], 1u << (i & 31)) >> (i & 31)) & 1u) << q;
        }
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
    const int whole_steps = N / PLAN_BLOCK;              // (uniform) steps in which every lane has a slot
#pragma unroll
    for (int q = 0; q < PLAN_IPT; ++q) {
        const int j = q * PLAN_BLOCK + tid;
        if (q < whole_steps || j < N) L.gpre[j] = L.wave_pref[q * PLAN_WAVES + w] + (inc[q] - len[q]);
    }
    __syncthreads();

    // ---- 2. shard bases: lane p takes shard p; exclusive scan of the loads rounded up to the alignment ----
    if (P <= WAVE) {                                     // (uniform) one wave holds every shard: no barrier, the others go on
        if (w == 0) {
            const int64_t first = lane < P ? L.gpre[L.shard_off[lane]] : 0;
            const int64_t load = lane < P ? L.gpre[L.shard_off[lane + 1]] - first : 0;
            const int64_t padded = a.align == 1 ? load : (load + a.align - 1) / a.align * a.align;   // (uniform)
            const int64_t inc = wave_incl_scan_add<int64_t>(padded);
            const int64_t end = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)((uint64_t)inc >> 32), WAVE - 1) << 32) |
                                          (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)inc, WAVE - 1));
            if (lane < P) { L.shard_base[lane] = inc - padded; a.shard_tok_off[lane] = inc - padded; }
            if (lane == 0) {
                L.shard_base[P] = end;
                a.shard_tok_off[P] = end;
                a.dst_tok_off[N] = end;
                if (end > a.capacity) set_status(a.status, DC_ERR_OVERFLOW);
            }
        }
    } else {
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
        // Few shards: a group of 32 or 16 LANES walks a shard (every wave takes 2 or 4 shards).  A
        // hop probes G slots at once, one per lane: the prefix sums do not decrease, so the lanes that still fit
        // are a prefix of the group and a ballot counts them - one LDS round trip per window where the
        // dependent probes of a bisection take six to eight.  (Not a whole wave per shard, even where there are
        // waves enough: a hop costs a wave the same instructions whatever its groups' width, sixteen waves
        // walking at once are bound by the compute unit's issue rate, and eight or fewer by a hop's latency,
        // which is the shorter of the two.)
        const int spw = P <= PLAN_WAVES ? 2 : 4;             // shards per wave
        const int G = WAVE / spw, g = lane / G, gl = lane - g * G;
        const int lg_G = spw == 2 ? 5 : 4;
        const uint64_t group_mask = (G == WAVE ? ~0ull : (1ull << G) - 1ull);
        const int p = w * spw + g;
        if (p < P) {
            const int b = L.shard_off[p + 1];
            int j = L.shard_off[p];
            int sz = 0;                                      // slots in the micro-batch before this one
            while (j < b) {                                  // uniform over the group
                if (gl == 0) atomicOr(&L.start_bits[j >> 5], 1u << (j & 31));
                const int64_t limit = L.gpre[j] + a.budget;
                // the last e in (j, b] with gpre[e] <= limit (j + 1 if there is none: an over-budget slot still
                // advances by one).  The first window probes G slots one by one, placed around the end that a micro-batch
                // as long as the one before would have (slots of a shard come in descending length, so it holds a few
                // more; the first one of a shard: the G slots behind the start).  Most micro-batches end inside it; if
                // not, the group's lanes spread evenly over what is left on the side where the end lies, then over the
                // stretch between the last probe that fits and the first that does not.
                const int first = max(j + 1, j + sz + 1 - (G >> 2));
                int lo, hi = b, e = j + 1;                   // candidates [lo, hi]; everything below lo fits
                {
                    const int c = first + gl;
                    const bool fits = c <= b && L.gpre[min(c, b)] <= limit;
                    const int cnt = __popcll((__ballot(fits) >> (g * G)) & group_mask);
                    if (cnt == 0) { lo = j + 1; hi = first - 1; }            // it ends before the window (or with its first slot)
                    else { e = first + cnt - 1; lo = (cnt == G && first + G <= b) ? first + G : b + 1; }     // b + 1: found
                }
                while (lo <= hi) {
                    const int S = (hi - lo + G) >> lg_G;     // ceil(candidates / G) >= 1
                    const bool fits = L.gpre[min(lo + (gl + 1) * S - 1, hi)] <= limit;
                    const int cnt = __popcll((__ballot(fits) >> (g * G)) & group_mask);
                    if (cnt > 0) e = min(lo + cnt * S - 1, hi);
                    if (cnt == G) break;                     // the last lane's probe is hi itself
                    hi = min(lo + (cnt + 1) * S - 1, hi) - 1;
                    lo += cnt * S;
                }
                sz = e - j;
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
    {   // (the two scans share their barriers)
        const uint32_t bits = tid < PLAN_WORDS ? L.start_bits[tid] : 0u;
        const int32_t n_here = (int32_t)__popc(bits), last_here = bits ? tid * 32 + 31 - __clz(bits) : -1;
        const int32_t inc_n = wave_incl_scan_add<int32_t>(n_here), inc_l = wave_incl_scan_max(last_here);
        int32_t* tmp_l = reinterpret_cast<int32_t*>(L.tmp64);
        if (lane == WAVE - 1) { L.tmp32[w] = inc_n; tmp_l[w] = inc_l; }
        __syncthreads();
        int32_t before = inc_n - n_here, last = wave_shift_up1(inc_l, -1);
        M = 0;
        for (int i = 0; i < PLAN_WAVES; ++i) {
            const int32_t x = L.tmp32[i];
            if (i < w) { before += x; last = max(last, tmp_l[i]); }
            M += x;
        }
        if (tid < PLAN_WORDS) { L.word_starts[tid] = before; L.word_last[tid] = last; }
        if (tid == 0) L.word_starts[PLAN_WORDS] = M;
    }
    __syncthreads();
    // One slot per lane and step.  Nothing here depends on a lane's own condition except the stores of a last,
    // partial step: every slot of a micro-batch stores the micro-batch's first slot (the same word with the same
    // value), and every slot stores the cu_seqlens entry behind its own, which is either the entry that the next
    // slot stores too or the end of the micro-batch.  Differences of prefix sums inside a micro-batch fit 32 bits,
    // so they are taken between the low words.
    const bool shift_bases = a.align != 1;               // (uniform)
    auto low_word = [&](int at) { return reinterpret_cast<const uint32_t*>(&L.gpre[at])[0]; };
    auto slot_out = [&](int q, bool whole) {             // whole (uniform): every lane has a slot in this step
        const int jr = q * PLAN_BLOCK + tid, j = whole ? jr : min(jr, N - 1);
        const uint32_t bits = L.start_bits[j >> 5];
        const uint32_t upto = bits & (0xFFFFFFFFu >> (31 - (j & 31)));               // starts at slots <= j of the word
        const int32_t m = L.word_starts[j >> 5] + (int32_t)__popc(upto) - 1;         // my micro-batch
        const int32_t first = upto ? (j & ~31) + 31 - __clz(upto) : L.word_last[j >> 5];     // its first slot (slot 0 starts one)
        const int64_t g = L.gpre[j];
        const uint32_t g_next = low_word(j + 1), g_first = low_word(max(first, 0));
        int64_t d = g;
        if (shift_bases) {                               // shard of the slot, then its aligned base
            int lo = 0, hi = P - 1;                      // largest p with shard_off[p] <= j
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (L.shard_off[mid] <= j) lo = mid; else hi = mid - 1;
            }
            d = g + (L.shard_base[lo] - L.gpre[L.shard_off[lo]]);
        }
        if (whole || jr < N) {
            a.dst_tok_off[(uint32_t)j] = d;
            a.mb_seq_off[(uint32_t)m] = first;
            a.cu_seqlens[(uint32_t)(j + m)] = (int32_t)((uint32_t)g - g_first);
            a.cu_seqlens[(uint32_t)(j + m) + 1u] = (int32_t)(g_next - g_first);
        }
    };
#pragma unroll 4
    for (int q = 0; q < whole_steps; ++q) slot_out(q, true);
    if (whole_steps < nb) slot_out(whole_steps, false);
    for (int p = tid; p <= P; p += PLAN_BLOCK) {         // micro-batches before each shard's first slot
        const int js = L.shard_off[p];
        int32_t c = M;
        if (js < N) c = L.word_starts[js >> 5] + (int32_t)__popc(L.start_bits[js >> 5] & ((1u << (js & 31)) - 1u));
        a.shard_mb_off[p] = c;
    }
    if (tid == 0) { *a.n_mb = M; a.mb_seq_off[M] = N; }
}

}  // namespace dc
