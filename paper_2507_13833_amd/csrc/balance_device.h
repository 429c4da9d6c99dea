// Device code of Algorithm 1 shared by the balance kernels (balance.hip: everything in the LDS;
// balance_large.hip: more sequences than the LDS holds): the workgroup's LDS layout, the stable counting
// pass of the radix sort, and the assignment rounds.
#pragma once
#include <cstddef>
#include "advantage_device.h"
#include "dc_lanes.h"

namespace dc {

constexpr int BAL_BLOCK = 1024;
constexpr int BAL_WAVES = BAL_BLOCK / WAVE;
// Row length of the sort's (digit, wave) counters: odd, so that the digits' rows start in different LDS banks.  (With
// rows of 16 words the 64 lanes of a wave, each at its own digit and all at the same wave index, met in two banks.)
constexpr int CNT_PITCH = BAL_WAVES + 1;
constexpr int BAL_ROUNDS = DC_MAX_SEQ / BAL_BLOCK;       // 64-item rounds per wave at the size limit
constexpr uint32_t KEY_FULL = 0xFFFFFFC0u;               // | worker id: full (or absent) worker

// When every partition ends with exactly C items its place in perm is known beforehand, and wave 0 files
// the items per worker (worker k's row starts at k * pitch) as it places them; the pitch is C rounded up
// to 2 mod 4, so that the 64 workers' rows start in 64 different LDS banks.
constexpr int PLACE_PAD = 4 * WAVE;
__device__ __forceinline__ int place_pitch(int C) { return C + ((2 - C) & 3); }

struct BalLds {
    int32_t  keys[DC_MAX_SEQ + PLACE_PAD];    // sequence lengths (sanitised); packed path: the sorted items, see lpt_rounds_packed
    alignas(16) uint32_t cnt[256 * CNT_PITCH];   // [digit][wave] counters of the sort passes; afterwards the workers' tables
                                              // (keys and cnt together: the bins of bin_sort_packed)
    uint16_t idx_a[DC_MAX_SEQ + PLACE_PAD];   // sort ping
    uint16_t idx_b[DC_MAX_SEQ + PLACE_PAD];   // sort pong; after the sort the free one holds every item's place in its
                                              // partition, or (all partitions of equal size) the partitions themselves
    int32_t  red[2 * BAL_WAVES];
    uint32_t tmp32[16];
    int32_t  spare[2];                    // where lanes without a worker put the stores of a round
    alignas(16) uint32_t nowhere[4];      // where a lane with nothing to store puts a 16-byte store
    int32_t  turn;                        // bin_sort_packed: the wave whose turn it is to count
    uint64_t tmp64[BAL_WAVES];
};
static_assert(sizeof(uint32_t) * 256 * BAL_WAVES >= 2 * sizeof(uint64_t) * DC_MAX_SHARDS, "two key tables fit the counters");
static_assert(DC_MAX_SHARDS <= BAL_BLOCK, "one thread per worker");

// Where the tables of the assignment live inside BalLds::cnt once the sort is done.
constexpr int PART_OFF_AT = 0;                         // int32 [P + 1]: start of every P_k inside perm
constexpr int PLACED_AT = DC_MAX_SHARDS + 8;           // int32: items placed
constexpr int WCOUNT_AT = DC_MAX_SHARDS + 16;          // int32 [64]: |P_k| of the one-wave path

// One stable counting pass over positions [0, N): position pos carries digit(pos) in
// [0, 256); emit(pos, out) receives its output position.  Wave w owns the contiguous
// positions [w*rounds*64, (w+1)*rounds*64), so (digit, wave, rank-in-wave) is the
// stable order.  Every lane of the workgroup must call it.
template <typename DigitFn, typename EmitFn>
__device__ __forceinline__ void counting_pass(BalLds& L, int N, int rounds, DigitFn digit, EmitFn emit) {
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    const int wave_base = w * rounds * WAVE;
    for (int i = tid; i < 256 * CNT_PITCH; i += BAL_BLOCK) L.cnt[i] = 0;
    __syncthreads();
    uint32_t packed[BAL_ROUNDS];                                  // digit << 16 | rank before me in my wave
#pragma unroll
    for (int r = 0; r < BAL_ROUNDS; ++r) {
        packed[r] = 0;
        if (r < rounds) {                                         // uniform
            const int pos = wave_base + r * WAVE + lane;
            const bool valid = pos < N;
            uint32_t d = 0;
            if (valid) d = digit(pos) & 0xFFu;
            // lanes holding my digit: for every bit, the lanes whose bit equals mine (an invalid lane has d = 0
            // and is not among the valid ones to begin with)
            const uint64_t valid_lanes = __builtin_amdgcn_ballot_w64(valid);
            uint32_t peers_lo = (uint32_t)valid_lanes, peers_hi = (uint32_t)(valid_lanes >> 32);
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const uint64_t bal = __builtin_amdgcn_ballot_w64(((d >> b) & 1u) != 0u);
                const uint32_t mine = (uint32_t)__builtin_amdgcn_sbfe((int)d, (unsigned)b, 1u);   // all ones if my bit is set
                peers_lo &= ~((uint32_t)bal ^ mine);
                peers_hi &= ~((uint32_t)(bal >> 32) ^ mine);
            }
            const uint64_t peers = ((uint64_t)peers_hi << 32) | peers_lo;
            const uint64_t lt = (1ull << lane) - 1ull;
            const int before = __popcll(peers & lt);
            const int leader = valid ? (__ffsll((long long)peers) - 1) : lane;
            uint32_t old = 0;
            if (valid && lane == leader) {                        // one lane per distinct digit
                uint32_t* c = &L.cnt[d * CNT_PITCH + w];
                old = *c;
                *c = old + (uint32_t)__popcll(peers);
            }
            old = (uint32_t)__shfl((int)old, leader, WAVE);
            packed[r] = (d << 16) | (old + (uint32_t)before);
        }
    }
    __syncthreads();
    {   // exclusive scan of the 4096 counters in (digit, wave) order: thread t takes digit t / 4, waves 4 (t % 4) ...
        static_assert(BAL_BLOCK * 4 == 256 * BAL_WAVES, "four counters per thread");
        uint32_t* mine = &L.cnt[(tid >> 2) * CNT_PITCH + (tid & 3) * 4];
        uint32_t c4[4], s = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) { c4[q] = mine[q]; s += c4[q]; }
        uint32_t tot;
        uint32_t run = block_excl_scan_add<uint32_t>(s, L.tmp32, &tot);
#pragma unroll
        for (int q = 0; q < 4; ++q) { mine[q] = run; run += c4[q]; }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < BAL_ROUNDS; ++r) {
        if (r < rounds) {
            const int pos = wave_base + r * WAVE + lane;
            if (pos < N) {
                const uint32_t d = packed[r] >> 16, rk = packed[r] & 0xFFFFu;
                emit(pos, (int)(L.cnt[d * CNT_PITCH + w] + rk));
            }
        }
    }
    __syncthreads();
}

// The packed items (length << 16 | index, one per sequence) in the order of Algorithm 1's sorted list, longest
// first and equal lengths by index, written to out[0, N) in ONE pass where the two passes of the radix sort
// each rank every item among its wave's 64 by eight ballots: a bin per length value (bin b = longest - length,
// 16 bits wide, two to a word, in the LDS that the rows of the workers take over afterwards) is counted by
// atomic adds whose return value is the item's ticket within its bin, the bins are scanned, and start + ticket
// is the item's place.  The order inside a run of one length is the order of the tickets.  The waves count one
// after the other, wave w holding the w-th stretch of the sequences, a wave's LDS operations execute in the
// order it issues them, and the adds of one instruction that meet in a word take effect in lane order: the last
// of these is what the chip is seen to do, not what it is documented to do, so the result is checked (two
// neighbours of one length in the wrong order, anywhere) and a list that fails is sorted by the radix passes
// like one that the bins do not serve.  false (and out[] undefined) in that case, and if some length occurs more
// than BIN_RUN_MAX times (adds that meet in one word take effect one by one): the caller then sorts by radix passes.
// range = longest - shortest, at most BIN_RANGE_MAX; the caller has zeroed the BIN_WORDS words from L.keys on
// and L.turn, with a barrier since.  Every lane of the workgroup must call it; len[q] = length of sequence
// bal_item(q, rounds), unchanged where the result is false and used up otherwise.
constexpr int BIN_WORDS = DC_MAX_SEQ + PLACE_PAD + 256 * CNT_PITCH;
constexpr int BIN_QUADS = (BIN_WORDS / 4 + BAL_BLOCK - 1) / BAL_BLOCK;      // 16-byte pieces of the bins per thread, at most
constexpr uint32_t BIN_RANGE_MAX = 2u * BIN_WORDS - 4u;
constexpr uint32_t BIN_RUN_MAX = 1024;
constexpr int BIN_SPINS = 1 << 16;                               // looks at the turn word before a wave stops waiting (the last wave needs ~30)
constexpr int BIN_GROUP = 4;                                      // items a thread handles as one straight piece of code
static_assert(offsetof(BalLds, cnt) == sizeof(int32_t) * (DC_MAX_SEQ + PLACE_PAD), "the counters follow the keys");
static_assert(DC_MAX_SEQ < (1 << 15), "a place, and the sum of the counts, fit 16 bits with room to spare");
static_assert(BAL_ROUNDS % BIN_GROUP == 0, "whole groups");

__device__ __forceinline__ void bin_sort_clear(BalLds& L) {
    static_assert(BIN_WORDS % 4 == 0 && offsetof(BalLds, keys) % 16 == 0, "whole 16-byte pieces");
    uint4* z = reinterpret_cast<uint4*>(L.keys);
    for (int j = threadIdx.x; j < BIN_WORDS / 4; j += BAL_BLOCK) z[j] = make_uint4(0u, 0u, 0u, 0u);
    if (threadIdx.x == 0) L.turn = 0;
}

// Which sequence a thread's q-th length register stands for: wave w holds the `rounds` * 64 consecutive sequences
// from w * rounds * 64 on, 64 of them per register, so that (wave, register, lane) order is index order.
__device__ __forceinline__ int bal_item(int q, int rounds) {
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    return (w * rounds + q) * WAVE + lane;
}

__device__ __forceinline__ bool bin_sort_packed(BalLds& L, int N, uint32_t longest, uint32_t range,
                                                int32_t (&len)[BAL_ROUNDS], uint32_t* out) {
    // The code below is laid out for the LDS's latency.  A thread's items go in groups of BIN_GROUP, a group being
    // one straight piece of code that issues all its LDS operations before it uses the first result, under a
    // uniform test of whether the group has items at all.  Inside a group no lane steps aside: a lane without an
    // item adds nothing, reads what a neighbour reads and writes to a spare word, because a branch on a lane's
    // own condition would end the straight piece.
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    uint32_t* bins = reinterpret_cast<uint32_t*>(L.keys);
    const int nw = (int)((range + 4u) >> 1);                      // bins 0 .. range, one more for the end of the last run
    const int rounds = (N + BAL_BLOCK - 1) / BAL_BLOCK;           // (uniform: the q that have items at all)
    // The count, wave after wave: a wave's LDS operations execute in the order it issues them, and the adds of one
    // instruction that meet in a word take effect in lane order (measured; nothing below relies on it, see the
    // check behind the scatter), so with the waves taking turns a bin's tickets rise with the sequence index and
    // every run of one length comes out of the scatter in index order.  A wave passes the turn on with a store
    // issued behind its adds, not behind their results.
    // One register per item: the length in the low half, the ticket above it.
    {
        // (what the adds need is worked out before the wave's turn comes: the turn itself is the adds and nothing else)
        uint32_t word[BAL_ROUNDS];                                // byte offset of the bin's word
        uint32_t old[BAL_ROUNDS];                                 // first what to add, then what the add returned
#pragma unroll
        for (int q = 0; q < BAL_ROUNDS; ++q) {
            const bool mine = q < rounds && bal_item(q, rounds) < N;
            const uint32_t b = mine ? longest - (uint32_t)len[q] : 0u;
            word[q] = 4u * (mine ? b >> 1 : (uint32_t)min(lane, nw - 1));
            old[q] = mine ? ((b & 1u) ? 0x10000u : 1u) : 0u;
            asm volatile("" : "+v"(word[q]), "+v"(old[q]));       // (here, not behind the wait)
        }
        const int wv = __builtin_amdgcn_readfirstlane(tid / WAVE);
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        // (the wait is bounded: a wave that gave up would count out of turn, which the check below would see)
        for (int spins = 0; spins < BIN_SPINS && __hip_atomic_load(&L.turn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < wv; ++spins)
            __builtin_amdgcn_s_sleep(1);
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        // (one straight run of adds, of all the registers or of their first half: a register without items adds nothing)
        auto add = [&](int q) { old[q] = atomicAdd(reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(bins) + word[q]), old[q]); };
        if (rounds > BAL_ROUNDS / 2) {
#pragma unroll
            for (int q = 0; q < BAL_ROUNDS; ++q) add(q);
        } else {
#pragma unroll
            for (int q = 0; q < BAL_ROUNDS / 2; ++q) add(q);
        }
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        if (lane == 0) __hip_atomic_store(&L.turn, wv + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
#pragma unroll
        for (int g = 0; g < BAL_ROUNDS; g += BIN_GROUP) {
            if (g < rounds) {
#pragma unroll
                for (int q = g; q < g + BIN_GROUP; ++q) {
                    const bool odd = ((longest - (uint32_t)len[q]) & 1u) != 0u;
                    len[q] |= (int32_t)(odd ? old[q] & 0xFFFF0000u : old[q] << 16);
                }
            }
        }
    }
    __syncthreads();
    // counts -> starts: a thread takes `per` consecutive 16-byte pieces (an odd number of them where that fits, for the banks)
    uint4* quads = reinterpret_cast<uint4*>(L.keys);
    const int nq = (nw + 3) >> 2;
    const int per = min(((nq + BAL_BLOCK - 1) / BAL_BLOCK) | 1, BIN_QUADS);
    const int lo = tid * per;
    uint4 w[BIN_QUADS];
#pragma unroll
    for (int k = 0; k < BIN_QUADS; ++k) w[k] = quads[min(lo + k, BIN_WORDS / 4 - 1)];
    uint32_t sum = 0, big = 0;
#pragma unroll
    for (int k = 0; k < BIN_QUADS; ++k) {
        if (!(k < per && lo + k < nq)) w[k] = make_uint4(0u, 0u, 0u, 0u);      // (bins beyond the last one hold zero already)
        const uint32_t x[4] = {w[k].x, w[k].y, w[k].z, w[k].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            sum += (x[c] & 0xFFFFu) + (x[c] >> 16);
            big = max(big, max(x[c] & 0xFFFFu, x[c] >> 16));
        }
    }
    uint32_t total;                                               // (a run above the limit rides the scan's high bits)
    uint32_t run = block_excl_scan_add<uint32_t>(sum | (big > BIN_RUN_MAX ? 1u << 20 : 0u), L.tmp32, &total) & 0xFFFFFu;
    if (total >> 20) {                                            // (uniform)
#pragma unroll
        for (int q = 0; q < BAL_ROUNDS; ++q) len[q] &= 0xFFFF;
        return false;
    }
    uint4* const nowhere = reinterpret_cast<uint4*>(L.nowhere);
#pragma unroll
    for (int k = 0; k < BIN_QUADS; ++k) w[k] = quads[min(lo + k, BIN_WORDS / 4 - 1)];      // (read again rather than kept: registers)
#pragma unroll
    for (int k = 0; k < BIN_QUADS; ++k) {
        const uint32_t x[4] = {w[k].x, w[k].y, w[k].z, w[k].w};
        uint32_t y[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t c0 = x[c] & 0xFFFFu;
            y[c] = run | ((run + c0) << 16);
            run += c0 + (x[c] >> 16);
        }
        *((k < per && lo + k < nq) ? quads + lo + k : nowhere) = make_uint4(y[0], y[1], y[2], y[3]);
    }
    __syncthreads();
    auto run_of = [&](uint32_t b) {                               // start of the run of bin b | its size << 16
        const uint32_t wa = bins[b >> 1], wb = bins[(b >> 1) + 1];
        const uint32_t start = (b & 1u) ? wa >> 16 : wa & 0xFFFFu;
        return start | ((((b & 1u) ? wb & 0xFFFFu : wa >> 16) - start) << 16);
    };
    static_assert(128 + 1 <= PLACE_PAD, "the zeroed words and the spare word lie in the array's padding");
#pragma unroll
    for (int g = 0; g < BAL_ROUNDS; g += BIN_GROUP) {
        if (g < rounds) {
            uint32_t at[BIN_GROUP];
#pragma unroll
            for (int q = g; q < g + BIN_GROUP; ++q) {
                const bool mine = q < rounds && bal_item(q, rounds) < N;
                at[q - g] = run_of(mine ? longest - ((uint32_t)len[q] & 0xFFFFu) : 0u);
            }
#pragma unroll
            for (int q = g; q < g + BIN_GROUP; ++q) {
                const int i = bal_item(q, rounds);
                const uint32_t to = (at[q - g] & 0xFFFFu) + ((uint32_t)len[q] >> 16);
                out[(q < rounds && i < N) ? to : (uint32_t)N + 128u] = ((uint32_t)len[q] << 16) | (uint32_t)i;
            }
        }
    }
    out[N + (tid & 127)] = 0;
    __syncthreads();
    // Is every run in index order?  (A thread looks at places q * BAL_BLOCK + tid here, not at its sequences; a
    // place beyond the last one repeats the last one's work.)
    {
        bool wrong = false;
#pragma unroll
        for (int g = 0; g < BAL_ROUNDS; g += BIN_GROUP) {
            if (g < rounds) {
#pragma unroll
                for (int q = g; q < g + BIN_GROUP; ++q) {
                    const int at = min(q * BAL_BLOCK + tid, N - 1);
                    const uint32_t a = out[at], b = out[at + 1];
                    wrong |= ((a ^ b) < 0x10000u) && a > b;
                }
            }
        }
        const bool here = __ballot(wrong) != 0ull;
        if (lane == 0) L.red[tid / WAVE] = here ? 1 : 0;
        __syncthreads();
        int any = 0;
#pragma unroll
        for (int i = 0; i < BAL_WAVES; ++i) any |= L.red[i];
        if (!any) return true;                                    // (uniform)
    }
#pragma unroll
    for (int q = 0; q < BAL_ROUNDS; ++q) len[q] &= 0xFFFF;
    return false;
}

// The assignment rounds (wave 0 only).  WIDTH = 16, 32 or 64 >= P lanes take part in the sort.
// pitch == 0: step_slot[t] = place of item I[t] inside its worker's partition; pitch > 0 (every
// partition will hold exactly C items): step_slot[k * pitch + c] = the c-th item of worker k.
// The worker of a placed sequence takes the place of its length in keys[] (an item's length is
// read for the last time before the item is placed); worker_count[k] = |P_k|.  Returns the number of
// items placed (N).
// What the rounds keep per worker (lane k: worker k) from one call to the next when the items arrive
// in several portions (a round is a run of consecutive pop-mins of Algorithm 1, so the item stream may
// be cut anywhere).
struct LptCarry {
    uint32_t key;
    int32_t  count;
    int64_t  load;
    bool     all_take;
};
__device__ __forceinline__ LptCarry lpt_fresh(int P, int C) {
    const uint32_t lane = threadIdx.x;
    LptCarry c;
    c.key = ((int)lane < P && C > 0) ? lane : (KEY_FULL | lane);
    c.count = 0;
    c.load = 0;
    c.all_take = C > 0;
    return c;
}

// TIGHT: P == WIDTH and pitch > 0 (the printed algorithm on 16, 32 or 64 workers): the rounds in which every
// worker takes an item drop the selects that the general case needs.
template <int WIDTH, bool TIGHT = false>
__device__ __forceinline__ int lpt_rounds(int N, int P, int C, int32_t* keys, const uint16_t* sorted,
                                          int32_t max_len, uint16_t* step_slot, int pitch, int32_t* spare_word,
                                          int32_t* worker_count, int64_t* __restrict__ shard_load, LptCarry& carry) {
    const uint32_t lane = threadIdx.x;
    // Keys of open workers lie within one longest sequence (G, in key units) of the smallest, which
    // grows by at most G per round.  A check that leaves the smallest below 2^30 therefore keeps every
    // key below 2^30 + (R + 1) G for the next R rounds; R is chosen so that this stays below 2^32
    // with one G to spare.
    const uint32_t G = (uint32_t)__builtin_amdgcn_readfirstlane(max_len) << 6;    // max_len <= 2^24
    const uint32_t fit = (3u << 30) / max(G, 1u);                 // >= 3
    const int check_every = (int)min(64u, fit - 2u);
    int until_check = 1;
    const uint32_t full = KEY_FULL | lane;
    const bool mine_exists = (int)lane < P;                       // lane k keeps worker k
    const uint64_t everyone = P == WAVE ? ~0ull : (1ull << P) - 1ull;
    uint32_t key = carry.key;
    int32_t count = carry.count;
    int64_t load = carry.load;
    int pos = 0;
    // the item offered to rank `lane` is fetched one round ahead (two dependent LDS reads), as soon as the
    // accepted prefix is known, so the reads overlap the hand-back of the keys instead of delaying the sort
    uint32_t idx = N > 0 ? (uint32_t)sorted[min((int)lane, N - 1)] : 0u;
    uint32_t s = N > 0 ? (uint32_t)keys[idx] : 0u;
    bool all_take = carry.all_take;                               // every worker open and the last round placed an item on each

    while (pos < N) {
        // ---- rounds in which every worker takes one item ----
        // While all P workers are open and whole prefixes are accepted, a worker's count is its count at
        // entry plus the rounds since, and its load is its key plus a constant.  Nothing has to travel back
        // to the worker lanes then: the keys stay in rank order from round to round, and the sort of the
        // updated keys starts before the round's acceptance test has finished (it is only used if the
        // test passes), which takes the test off the chain of dependent sorts.
        if (all_take && pos + P <= N) {                           // uniform
            uint32_t cmax = mine_exists ? (uint32_t)count : 0u;
            wave_all_reduce([&](auto j) { cmax = max(cmax, lane_xor<decltype(j)::value>(cmax)); });
            const int avail = C - __builtin_amdgcn_readfirstlane((int)cmax);   // rounds before the first worker is full (>= 1)
            const int64_t off = load - (int64_t)(key >> 6);       // what the key does not hold of my worker's load
            int64_t taken = 0;                                    // load taken off the keys by rebasing in here
            int rounds = 0;
            uint32_t sk = wave_sort_asc<WIDTH>(key);
            // items two rounds ahead: nothing a round reads from LDS depends on what the round computes
            uint32_t idx1 = sorted[min(pos + P + (int)lane, N - 1)];
            // every LDS read issued so far is waited for here, outside the loop: a wait left to the loop's
            // first use would sit in the loop and also wait, every round, for the stores of the round before
            asm volatile("" : "+v"(idx1), "+v"(s), "+v"(idx));
            // The two LDS stores that record a round's placements are issued at the top of the NEXT round,
            // behind that round's reads.  LDS operations retire through one in-order counter and the compiler
            // waits for "everything" at the loop's joins, so a round's first wait also waits for the stores
            // before it: placed here they have a whole sort to retire, placed at the round's end they
            // stall the next round.  Lanes without a worker store to spare words (no branch round the stores).
            uint32_t st_slot = DC_MAX_SEQ + PLACE_PAD - 1, st_val = 0, st_id = 0;      // nothing to record yet
            int32_t* st_key = spare_word;
            const int n_rounds = min(avail, (N - pos) / P);       // >= 1: until a worker is full or the items run out
            while (rounds < n_rounds) {
                if (__builtin_expect(--until_check == 0, 0)) {    // uniform; first, so that the rest of the round is one
                    until_check = check_every;                    // straight run of instructions for the scheduler
                    const uint32_t min0 = (uint32_t)__builtin_amdgcn_readlane((int)sk, 0);
                    if (min0 >= 0x40000000u && min0 < KEY_FULL) {
                        const uint32_t sub = min0 & ~63u;
                        if (sk < KEY_FULL) sk -= sub;
                        taken += (int64_t)(sub >> 6);
                    }
                }
                const int t = pos + (int)lane;                    // rank `lane` takes item I[t]
                const uint32_t id = sk & 63u;
                const uint32_t s1 = (uint32_t)keys[idx1];
                const uint32_t idx2 = sorted[min(t + 2 * P, N - 1)];
                const int32_t before = __builtin_amdgcn_ds_bpermute((int)(id << 2), count) + rounds;   // its count
                step_slot[st_slot] = (uint16_t)st_val;            // the round before: place inside the partition ...
                *st_key = (int32_t)st_id;                         // ... and worker (the item's length is not needed again)
                // absent workers keep their all-ones-ish key; with WIDTH workers the lanes beyond them sort among
                // themselves and come behind them in the scan: what they hold does not matter
                const uint32_t newk = (TIGHT || mine_exists) ? sk + (s << 6) : sk;
                // next round's order, if this round stands; the acceptance test is computed between the steps of
                // the sort's first levels (the last level is made to wait for its result)
                const uint32_t half_sorted = wave_sort_front<WIDTH>(newk);
                const uint32_t pm = wave_excl_scan_umin((TIGHT || mine_exists) ? newk : 0xFFFFFFFFu);
                const uint64_t takers = __builtin_amdgcn_ballot_w64(sk < pm);
                const bool refused = (takers & everyone) != everyone;
                const uint32_t sk2 = wave_sort_back<WIDTH>(half_sorted, (uint32_t)refused);
                if (__builtin_expect(refused, 0)) break;          // not everyone's turn: one general round
                constexpr bool EVERY_LANE = TIGHT && WIDTH == WAVE;           // every lane keeps a worker
                const int slot_at = (TIGHT || pitch) ? (int)id * pitch + before : t;
                st_slot = (EVERY_LANE || mine_exists) ? (uint32_t)slot_at : (uint32_t)(DC_MAX_SEQ + PLACE_PAD - 1);
                st_val = (TIGHT || pitch) ? idx : (uint32_t)before;
                st_key = (EVERY_LANE || mine_exists) ? keys + idx : spare_word;
                st_id = id;
                pos += P;
                rounds += 1;
                sk = sk2;
                idx = idx1;
                s = s1;
                idx1 = idx2;
            }
            // the last accepted round's record (after a refused round: the same stores once more)
            step_slot[st_slot] = (uint16_t)st_val;
            *st_key = (int32_t)st_id;
            // back to worker lanes: rank r sends its key to lane (sk & 63); absent workers send theirs to themselves
            if (TIGHT && !mine_exists) sk = full;                 // (whatever the rounds left in their lanes)
            key = (uint32_t)__builtin_amdgcn_ds_permute((int)((sk & 63u) << 2), (int)sk);
            if (mine_exists) {
                count += rounds;
                load = off + taken + (int64_t)(key >> 6);
                if (count == C) key = full;
            }
            until_check = 1;
            all_take = false;
            continue;
        }

        // ---- a general round: the longest accepted prefix of the ranks takes one item each ----
        const int t = pos + (int)lane;
        uint32_t sk = wave_sort_asc<WIDTH>(key);                  // lane r: r-th smallest key
        if (--until_check == 0) {                                 // uniform
            until_check = check_every;
            const uint32_t min0 = (uint32_t)__builtin_amdgcn_readlane((int)sk, 0);
            if (min0 >= 0x40000000u && min0 < KEY_FULL) {         // rebase: subtract the minimum load
                const uint32_t sub = min0 & ~63u;
                if (key < KEY_FULL) key -= sub;
                if (sk < KEY_FULL) sk -= sub;
            }
        }
        const bool valid = sk < KEY_FULL && t < N;
        const uint32_t newk = valid ? sk + (s << 6) : 0xFFFFFFFFu;
        const uint32_t pm = wave_excl_scan_umin(newk);            // smallest updated key among ranks below mine
        const uint64_t acc = __ballot(valid && sk < pm);
        const int m = (~acc == 0ull) ? WAVE : (__ffsll((long long)~acc) - 1);   // accepted prefix
        if (m == 0) break;                                        // cannot happen: cap * P >= N
        const uint32_t next_idx = sorted[min(t + m, N - 1)];      // next round's item: first read
        // back to worker lanes: rank r sends its updated key, its own rank in place of the worker id,
        // to lane (sk & 63)
        const uint32_t recv = (uint32_t)__builtin_amdgcn_ds_permute((int)((sk & 63u) << 2), (int)((newk & ~63u) | lane));
        const uint32_t thr = (uint32_t)__builtin_amdgcn_readlane((int)sk, m - 1);
        const uint32_t next_s = (uint32_t)keys[next_idx];         // second read
        if (key <= thr) {                                         // my worker is among the m smallest
            const uint32_t nk = (recv & ~63u) | lane;
            const int mine = pos + (int)(recv & 63u);             // the item I took
            const uint32_t u_mine = sorted[mine];
            if (pitch) step_slot[(int)lane * pitch + count] = (uint16_t)u_mine;
            else step_slot[mine] = (uint16_t)count;
            keys[u_mine] = (int32_t)lane;                     // the item is placed: its length is not needed again
            load += (int64_t)((nk - key) >> 6);
            count += 1;
            key = (count == C) ? full : nk;
        }
        pos += m;
        idx = next_idx;
        s = next_s;
        all_take = m == P && __ballot(mine_exists && key >= KEY_FULL) == 0ull;
    }
    if (mine_exists) shard_load[lane] = load;
    worker_count[lane] = count;
    carry.key = key; carry.count = count; carry.load = load; carry.all_take = all_take;
    return pos;
}

// ---------------------------------------------------------------------------------------------------
// The rounds once more for the printed algorithm on up to 32 or on 64 workers (P <= WIDTH = 16 or 32, or P = 64; N == P * C) with
// lengths below 2^16: the common case, and the one in which the rounds are most of the kernel's time.
//
// A round of one wave is the sort of the 64 updated keys, a chain of dependent instructions with idle
// issue cycles between them, plus whatever else the round does.  Measured on the chip, vector
// instructions placed into those idle cycles are nearly free, but every LDS instruction costs the wave
// about 20 cycles, a scalar branch on a vector result 50 to 60 (the scalar unit waits for the vector
// pipeline), and the loop's own branch about 40.  So this path
//   - keeps the sorted items as ONE array of 32-bit words, length << 16 | sequence, in sorted order
//     (items[]; built by the whole workgroup after the sort): a round reads one word per lane at an address
//     that does not depend on anything it computes, instead of an index and then a length;
//   - files that whole word in its worker's row (rows[k * pitch + c] = the c-th item of worker k), so that no
//     second store per round records the worker of a sequence; the layout pass derives it from the row;
//   - takes the worker's count from a cross-lane read only when the workers' counts differ at the phase's
//     start (they do not unless rounds with fewer takers came before);
//   - runs FAST_BATCH rounds as one straight piece of code without a test when a bound says that all of
//     them will stand, and one round at a time with the exact test otherwise;
//   - finishes a round that fails the test where it stands, as a short round (the accepted prefix of the ranks
//     takes its items, the keys are sorted again, the workers that sat out are told so by one cross-lane write),
//     instead of sending the keys back to the workers' lanes for a general round and sorting them twice more
//     on the way back in.  While no worker is full a worker's place in its row is its place at the phase's
//     start plus the round number minus the rounds it sat out.
// The bound: keys come in ascending order and items in descending order.  With D = largest - smallest key,
// a round stands if D < its smallest item (the largest key is then below every updated key), and it leaves
// D' <= max(D, its largest - its smallest item).  So a run of rounds stands if D < L and F - L < L, where
// F = the first item of the run and L = its last one.  One look at 64 items (the last ones of the next 64
// batches, one per lane) says how many batches that covers: up to 256 rounds per look.
//
// PORTION: the N items are one portion of a longer sorted list (more sequences than the LDS holds).  The workers'
// keys, counts and loads come from, and go back to, *carry; the item words carry their index inside the portion;
// the rows start empty with every call and hold row_cap items each, and the call returns, before all N items are
// placed, as soon as one row is full (the caller empties the rows and offers the rest again).
constexpr int FAST_BATCH = 4;
constexpr uint32_t PACKED_MAX_LEN = 0xFFFFu;             // lengths up to this take the packed path

__device__ __forceinline__ int row_pitch(int C) { return C | 1; }      // odd: the workers' rows start in different banks

// What lane k keeps of worker k between two portions.
struct PackedCarry {
    uint32_t key;
    int32_t  count;
    int64_t  load;
};
__device__ __forceinline__ PackedCarry packed_fresh(int P, int C) {
    const uint32_t lane = threadIdx.x & (WAVE - 1);
    PackedCarry c;
    c.key = ((int)lane < P && C > 0) ? lane : (KEY_FULL | lane);
    c.count = 0;
    c.load = 0;
    return c;
}

template <int WIDTH, bool PORTION = false>
__device__ __forceinline__ int lpt_rounds_packed(int N, int P, int C, const uint32_t* items, int32_t max_len,
                                                 uint32_t* rows, int pitch, uint32_t* spare_word,
                                                 int32_t* worker_count, int64_t* __restrict__ shard_load,
                                                 PackedCarry* carry = nullptr, int row_cap = 0) {
    const uint32_t lane = threadIdx.x;
    const uint32_t G = (uint32_t)__builtin_amdgcn_readfirstlane(max_len) << 6;    // see lpt_rounds for the rebasing
    const uint32_t fit = (3u << 30) / max(G, 1u);
    const int check_every = (int)min(64u, fit - 2u);
    int until_check = 1;
    const uint32_t full = KEY_FULL | lane;
    const bool mine_exists = (int)lane < P;                       // lane k keeps worker k, and plays rank k of the sorted order
    // WIDTH 64: P == 64.  WIDTH 8, 16 and 32: any P <= WIDTH; the keys of the lanes without a worker sort behind the
    // workers' and must stay where they are, so what is offered to their ranks is nothing: those lanes read the
    // zero word behind the last item, round after round (a stride of their own, no instruction more per round).
    constexpr bool SOME = WIDTH != WAVE && !PORTION;
    const bool offers = !SOME || mine_exists;
    const int stride = offers ? P : 0;                            // from a rank's item of one round to its item of the next
    const uint64_t everyone = P == WAVE ? ~0ull : (1ull << P) - 1ull;
    constexpr bool EVERY_LANE = WIDTH == WAVE;
    constexpr int NS = net_steps(WIDTH);
    constexpr int LAST = 2 * NS - 1;                              // the last gap of the sort (what an 8-lane sort has no later gap for goes there)
    static_assert(LAST >= 11, "the rounds' side work is laid out over twelve gaps at least");
    constexpr uint32_t NONE = 0xFFFFFFFFu;
    uint32_t key = (mine_exists && C > 0) ? lane : full;
    int32_t count = 0;
    int64_t load = 0;
    if constexpr (PORTION) { key = carry->key; count = carry->count; load = carry->load; }
    const int32_t row_base = count;                               // PORTION: my row's first entry is my item number row_base
    int pos = 0;
    uint32_t e = items[offers ? (int)lane : N];                   // the item offered to rank `lane` (the array is padded with zeros)
    bool all_take = C > 0;
    if constexpr (PORTION) all_take = __ballot(mine_exists && key >= KEY_FULL) == 0ull;
    const uint32_t pitch4 = (uint32_t)pitch * 4u;
    int no_look = 0, look_wait = 0;                               // tested rounds before the bound is looked at again
    char* const rows_b = reinterpret_cast<char*>(rows);
    char* const spare_b = reinterpret_cast<char*>(spare_word);

    while (pos < N) {
        if constexpr (PORTION) {                                  // a full row ends the portion
            if (__ballot(mine_exists && count - row_base >= row_cap) != 0ull) break;
        }
        if (all_take && pos + P <= N) {                           // uniform: every worker is open
            // (counts as the rows see them: PORTION counts from the call's start)
            const int32_t in_row = PORTION ? count - row_base : count;
            // (three butterflies of register exchanges, side by side: a shuffle through the LDS unit costs the lone
            //  wave its whole latency at each of the 6 dependent steps)
            uint32_t cmax = mine_exists ? (uint32_t)in_row : 0u, cmin = mine_exists ? (uint32_t)in_row : 0x7FFFFFFFu;
            uint32_t gmax = mine_exists ? (uint32_t)count : 0u;
            wave_all_reduce([&](auto j) {
                constexpr int J = decltype(j)::value;
                const uint32_t a = lane_xor<J>(cmax), b = lane_xor<J>(cmin);
                cmax = max(cmax, a);
                cmin = min(cmin, b);
                if constexpr (PORTION) gmax = max(gmax, lane_xor<J>(gmax));
            });
            const int c_hi = __builtin_amdgcn_readfirstlane((int)cmax), c_lo = __builtin_amdgcn_readfirstlane((int)cmin);
            bool level = c_hi == c_lo;                            // every row holds the same number of items (until a short round)
            const int64_t off = load - (int64_t)(key >> 6);       // what the key does not hold of my worker's load
            int64_t taken = 0;                                    // load taken off the keys by rebasing in here
            int rounds = 0;
            uint32_t sk = wave_sort_asc<WIDTH>(key);
            // >= 1: until a worker (PORTION: or a row) is full or the items run out
            const int n_rounds = PORTION ? min(min(C - __builtin_amdgcn_readfirstlane((int)gmax), row_cap - c_hi), (N - pos) / P)
                                         : min(C - c_hi, (N - pos) / P);
            const uint32_t* next_item = offers ? items + pos + P + (int)lane : items + N;      // the item of the next round for this rank
            int32_t count4 = in_row * 4;                          // lane k: 4 x (worker k's place in its row at round 0 of the phase)
            uint64_t refused_acc = 0;                             // ranks a refused round would have accepted

            // One round that is known to stand; r = rounds done before it in this phase.  LEVEL: all counts are c_lo.
            auto sure_round = [&](int r, auto level_c) {
                constexpr bool LEVEL = decltype(level_c)::value;
                uint32_t v = sk + ((e >> 16) << 6);               // the keys after this round
                const uint32_t id = sk & 63u;                     // the worker rank `lane` belongs to
                uint32_t e1 = 0;
                int32_t before4 = 0;
                const uint32_t row_at = 4u * (uint32_t)(LEVEL ? c_lo + r : r);
                v = wave_sort_steps<WIDTH, 0, NS>(v, [&](auto slot) {
                    constexpr int S = decltype(slot)::value;
                    if constexpr (S == 0) e1 = *next_item;
                    if constexpr (S == 1 && !LEVEL) before4 = __builtin_amdgcn_ds_bpermute((int)(id << 2), count4);
                    if constexpr (S == 3) next_item += stride;
                    if constexpr (S == 8) {
                        char* at = rows_b + (__umul24(id, pitch4) + (uint32_t)before4 + row_at);
                        if constexpr (!EVERY_LANE) at = mine_exists ? at : spare_b;
                        *reinterpret_cast<uint32_t*>(at) = e;      // filed with its worker
                    }
                    if constexpr (S == (LAST < 12 ? LAST : 12)) e = e1;
                });
                sk = v;
            };
            // One round with the exact test (every rank's key below the smallest updated key of the ranks before
            // it); false, and nothing changed but refused_acc, if it does not stand.  The row entry is written before
            // the outcome is known: a worker that does not take the item files its next one in the same place.
            auto tested_round = [&](int r) -> bool {
                const uint32_t sk_in = sk, e_in = e;
                uint32_t v = sk + ((e >> 16) << 6);
                uint32_t m = v;                                   // becomes the running minimum of the updated keys
                const uint32_t id = sk & 63u;
                uint32_t e1 = 0;
                int32_t before4 = 0;
                v = wave_sort_steps<WIDTH, 0, NS>(v, [&](auto slot) {
                    constexpr int S = decltype(slot)::value;
                    if constexpr (S == 0) e1 = *next_item;
                    if constexpr (S == 1) before4 = __builtin_amdgcn_ds_bpermute((int)(id << 2), count4);
                    if constexpr (S == 3) m = umin32(m, dpp_mov<DPP_ROW_SHR1>(NONE, m));
                    if constexpr (S == 5) m = umin32(m, dpp_mov<DPP_ROW_SHR2>(NONE, m));
                    if constexpr (S == 6) m = umin32(m, dpp_mov<DPP_ROW_SHR4>(NONE, m));
                    if constexpr (S == 7) m = umin32(m, dpp_mov<DPP_ROW_SHR8>(NONE, m));
                    if constexpr (S == 8) m = umin32(m, dpp_mov<DPP_ROW_BCAST15, 0xA>(NONE, m));
                    if constexpr (S == 9) m = umin32(m, dpp_mov<DPP_ROW_BCAST31, 0xC>(NONE, m));
                    if constexpr (S == 10) {
                        char* at = rows_b + (__umul24(id, pitch4) + (uint32_t)before4 + 4u * (uint32_t)r);
                        if constexpr (!EVERY_LANE) at = mine_exists ? at : spare_b;
                        *reinterpret_cast<uint32_t*>(at) = e;
                    }
                    if constexpr (S == 11) m = dpp_mov<DPP_WAVE_SHR1>(NONE, m);
                    if constexpr (S == (LAST < 13 ? LAST : 13)) e = e1;
                });
                const uint64_t acc = __ballot(sk_in < m) & everyone;
                if (__builtin_expect(acc != everyone, 0)) { e = e_in; refused_acc = acc; return false; }
                next_item += stride;
                sk = v;
                return true;
            };
            // What a refused round turns into: the longest accepted prefix of the ranks takes the items the refused
            // round offered them (its row entries are written already), the other workers stay where they are, and
            // the phase goes on: a worker's place in its row falls one behind the round number for every round it
            // sits out (count4, told to the worker's lane), and the next round's items start behind the ones taken.
            auto short_round = [&]() {
                const int took = __ffsll((long long)~refused_acc) - 1;     // >= 1: the lowest rank always takes
                const bool take = (int)lane < took;
                uint32_t v = take ? sk + ((e >> 16) << 6) : sk;
                const uint32_t to = mine_exists ? (sk & 63u) : lane;        // lanes without a worker talk to themselves
                const uint32_t* const at = offers ? items + pos + took + (int)lane : items + N;      // (the array is padded)
                uint32_t e1 = 0;
                int32_t behind4 = 0;
                v = wave_sort_steps<WIDTH, 0, NS>(v, [&](auto slot) {
                    constexpr int S = decltype(slot)::value;
                    if constexpr (S == 0) e1 = *at;
                    if constexpr (S == 1) behind4 = __builtin_amdgcn_ds_permute((int)(to << 2), take ? 0 : 4);
                    if constexpr (S == (LAST < 12 ? LAST : 12)) { count4 -= behind4; e = e1; }
                });
                sk = v;
                next_item = at + stride;
                pos += took;
            };

            while (rounds < n_rounds) {
                if (--until_check <= 0) {                         // uniform; every check_every rounds or so
                    until_check = check_every;
                    const uint32_t min0 = (uint32_t)__builtin_amdgcn_readlane((int)sk, 0);
                    if (min0 >= 0x40000000u && min0 < KEY_FULL) { // rebase: subtract the minimum load
                        const uint32_t sub = min0 & ~63u;
                        if (sk < KEY_FULL) sk -= sub;
                        taken += (int64_t)(sub >> 6);
                    }
                }
                // How many batches does the bound cover?  It asks for L > max(D / 64, F / 2) (D in key units); lane i
                // looks at the last item of the (i + 1)-th batch from here, and the items only get shorter.
                int sure = 0;
                const int may = min(n_rounds - rounds, until_check) / FAST_BATCH;      // batches before the phase ends / the next check
                if (may > 0 && --no_look < 0) {
                    const uint32_t k_lo = (uint32_t)__builtin_amdgcn_readlane((int)sk, 0);
                    const uint32_t k_hi = (uint32_t)__builtin_amdgcn_readlane((int)sk, P - 1);        // (the workers' largest)
                    const uint32_t first = (uint32_t)__builtin_amdgcn_readlane((int)e, 0) >> 16;
                    const uint32_t need = max((k_hi - k_lo) >> 6, first >> 1);
                    const uint32_t probe = items[min(pos + ((int)lane + 1) * (FAST_BATCH * P) - 1, N - 1)] >> 16;
                    const uint64_t good = __ballot((int)lane < may && probe > need);
                    sure = (~good == 0ull) ? WAVE : (__ffsll((long long)~good) - 1);
                    // a look costs about half a round: where the bound does not hold (one worker far above the
                    // others, as after a very long sequence) the next look waits, longer every time
                    look_wait = sure > 0 ? 0 : min(2 * look_wait + 2, 32);
                    no_look = look_wait;
                }
                if (sure > 0) {
                    if (level) {
                        for (int b = 0; b < sure; ++b) {
#pragma unroll
                            for (int u = 0; u < FAST_BATCH; ++u) sure_round(rounds + u, std::true_type{});
                            rounds += FAST_BATCH;
                        }
                    } else {
                        for (int b = 0; b < sure; ++b) {
#pragma unroll
                            for (int u = 0; u < FAST_BATCH; ++u) sure_round(rounds + u, std::false_type{});
                            rounds += FAST_BATCH;
                        }
                    }
                    until_check -= sure * FAST_BATCH - 1;
                    pos += sure * FAST_BATCH * P;
                } else {
                    // rounds with the exact test, in a loop of their own, until the next look or check
                    int burst = max(1, min(min(n_rounds - rounds, until_check), no_look + 1));
                    const int want = burst;
                    do {
                        if (tested_round(rounds)) pos += P;
                        else { short_round(); level = false; }
                        rounds += 1;
                    } while (--burst > 0);
                    until_check -= (want - burst) - 1;            // (one was taken off at the loop's top)
                    no_look -= want - burst;
                }
            }
            // back to worker lanes: rank r sends its key to lane (sk & 63); lanes without a worker send theirs to themselves
            if (!mine_exists) sk = full;                          // (whatever the rounds left in their lanes)
            key = (uint32_t)__builtin_amdgcn_ds_permute((int)((sk & 63u) << 2), (int)sk);
            if (mine_exists) {
                count = (count4 >> 2) + rounds + (PORTION ? row_base : 0);      // one item per round but the ones sat out
                load = off + taken + (int64_t)(key >> 6);
                if (count == C) key = full;
            }
            until_check = 1;
            all_take = false;
            continue;                                             // (rounds >= 1: a worker is full now, or the items have run out)
        }

        // ---- a general round: the longest accepted prefix of the ranks takes one item each ----
        const int t = pos + (int)lane;
        uint32_t sk = wave_sort_asc<WIDTH>(key);                  // lane r: r-th smallest key
        if (--until_check <= 0) {                                 // uniform
            until_check = check_every;
            const uint32_t min0 = (uint32_t)__builtin_amdgcn_readlane((int)sk, 0);
            if (min0 >= 0x40000000u && min0 < KEY_FULL) {         // rebase: subtract the minimum load
                const uint32_t sub = min0 & ~63u;
                if (key < KEY_FULL) key -= sub;
                if (sk < KEY_FULL) sk -= sub;
            }
        }
        const bool valid = sk < KEY_FULL && t < N;
        const uint32_t newk = valid ? sk + ((e >> 16) << 6) : 0xFFFFFFFFu;
        const uint32_t pm = wave_excl_scan_umin(newk);            // smallest updated key among ranks below mine
        const uint64_t acc = __ballot(valid && sk < pm);
        const int m = (~acc == 0ull) ? WAVE : (__ffsll((long long)~acc) - 1);   // accepted prefix
        if (m == 0) break;                                        // cannot happen: C * P == N
        // back to worker lanes: rank r sends its updated key, its own rank in place of the worker id,
        // to lane (sk & 63)
        const uint32_t recv = (uint32_t)__builtin_amdgcn_ds_permute((int)((sk & 63u) << 2), (int)((newk & ~63u) | lane));
        const uint32_t thr = (uint32_t)__builtin_amdgcn_readlane((int)sk, m - 1);
        const uint32_t next_e = items[t + m];                     // next round's item (padded array)
        if (key <= thr) {                                         // my worker is among the m smallest
            const uint32_t nk = (recv & ~63u) | lane;
            rows[(int)lane * pitch + (PORTION ? count - row_base : count)] = items[pos + (int)(recv & 63u)];     // the item I took
            load += (int64_t)((nk - key) >> 6);
            count += 1;
            key = (count == C) ? full : nk;
        }
        pos += m;
        e = offers ? next_e : 0u;
        all_take = __ballot(mine_exists && key >= KEY_FULL) == 0ull;      // every worker is open: the next round is tried above
    }
    if (mine_exists) shard_load[lane] = load;
    worker_count[lane] = count;
    if constexpr (PORTION) { carry->key = key; carry->count = count; carry->load = load; }
    return pos;
}

// The same rounds for 64 < P <= DC_MAX_SHARDS workers, run by the whole workgroup: thread k keeps
// worker k (64-bit key load << 10 | k, all-ones-ish when full or absent), thread r also plays
// rank r of the sorted order.  Every thread of the workgroup must call it (barriers inside).
// Returns the number of items placed; part_off[0..P] gets the start of every P_k.
constexpr int WIDE_ID_BITS = 10;
constexpr uint64_t WIDE_ID_MASK = (1ull << WIDE_ID_BITS) - 1ull;
constexpr uint64_t WIDE_FULL = ~WIDE_ID_MASK;          // | worker id: full (or absent) worker
static_assert(DC_MAX_SHARDS <= (1 << WIDE_ID_BITS), "worker id fits the key's low bits");

__device__ __forceinline__ uint64_t umin64(uint64_t a, uint64_t b) { return a < b ? a : b; }

// What thread k keeps of worker k between two portions of the items (see LptCarry).
struct WideCarry {
    uint64_t key;
    int32_t  count;
    int64_t  load;
};
__device__ __forceinline__ WideCarry wide_fresh(int P, int C) {
    const int tid = threadIdx.x;
    WideCarry c;
    c.key = (tid < P && C > 0) ? (uint64_t)tid : (WIDE_FULL | (uint64_t)tid);
    c.count = 0;
    c.load = 0;
    return c;
}

// The rounds over the N items of one portion.  Returns the number of items placed.
__device__ __forceinline__ int lpt_rounds_wide_portion(BalLds& L, int N, int P, int C, const uint16_t* sorted,
                                                       uint16_t* step_slot, WideCarry& carry) {
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    uint64_t* kbuf = reinterpret_cast<uint64_t*>(L.cnt);              // keys in worker order; then the keys sent back
    uint64_t* sbuf = kbuf + DC_MAX_SHARDS;                            // keys in rank order
    const uint64_t full = WIDE_FULL | (uint64_t)tid;
    uint64_t key = carry.key;
    int32_t count = carry.count;
    int64_t load = carry.load;
    int pos = 0;
    while (pos < N) {                                                 // pos is the same in every thread
        kbuf[tid] = key;
        __syncthreads();
        // my rank = keys below mine (keys are distinct: the worker id sits in the low bits)
        if (tid < P) {
            int rank = 0;
            for (int j = 0; j < P; ++j) rank += kbuf[j] < key ? 1 : 0;
            sbuf[rank] = key;
        }
        __syncthreads();
        // ---- rank view: thread r offers item I[pos + r] to the worker with the r-th smallest key ----
        const uint64_t sk = tid < P ? sbuf[tid] : ~0ull;
        const int t = pos + tid;
        const bool valid = tid < P && sk < WIDE_FULL && t < N;
        const uint64_t s = valid ? (uint64_t)(uint32_t)L.keys[sorted[t]] : 0ull;
        const uint64_t newk = valid ? sk + (s << WIDE_ID_BITS) : ~0ull;
        // smallest updated key among the ranks below mine
        uint64_t inc = newk;
#pragma unroll
        for (int d = 1; d < WAVE; d <<= 1) {
            const uint64_t o = __shfl_up(inc, d, WAVE);
            if (lane >= d) inc = umin64(inc, o);
        }
        uint64_t pm = __shfl_up(inc, 1, WAVE);
        if (lane == 0) pm = ~0ull;
        if (lane == WAVE - 1) L.tmp64[w] = inc;
        __syncthreads();
        for (int q = 0; q < w; ++q) pm = umin64(pm, L.tmp64[q]);
        // accepted prefix: ranks below the first one whose worker is no longer the minimum
        const uint64_t fail = __ballot(!(valid && sk < pm));
        if (lane == 0) L.red[w] = fail ? w * WAVE + (__ffsll((long long)fail) - 1) : BAL_BLOCK;
        __syncthreads();
        int m = BAL_BLOCK;
        for (int q = 0; q < BAL_WAVES; ++q) m = min(m, L.red[q]);
        if (m == 0) break;                                            // cannot happen: cap * P >= N (uniform)
        // back to the workers: rank r sends its updated key, its own rank in place of the worker id
        if (tid < m) kbuf[sk & WIDE_ID_MASK] = (newk & ~WIDE_ID_MASK) | (uint64_t)tid;
        const uint64_t thr = sbuf[m - 1];
        __syncthreads();
        if (tid < P && key <= thr) {                                  // my worker is among the m smallest
            const uint64_t recv = kbuf[tid];
            const uint64_t nk = (recv & ~WIDE_ID_MASK) | (uint64_t)tid;
            const int mine = pos + (int)(recv & WIDE_ID_MASK);        // the item I took
            step_slot[mine] = (uint16_t)count;
            L.keys[sorted[mine]] = tid;                               // placed: its length is not needed again
            load += (int64_t)((nk - key) >> WIDE_ID_BITS);
            count += 1;
            key = (count == C) ? full : nk;
        }
        pos += m;
        // the next round's first barrier separates these reads of kbuf from its rewriting by other threads:
        // a thread only overwrites its own entry before that barrier
    }
    carry.key = key; carry.count = count; carry.load = load;
    return pos;
}

// The same portion with lengths below 2^16 (max_len <= PACKED_MAX_LEN): 32-bit keys, (load - base) << 10 | k with
// the base taken off whenever the smallest key has passed 2^30 (open workers lie within one longest sequence of the
// smallest, a round adds at most one more, so the keys stay below 2^32: see lpt_rounds), and the ranks are found
// without looking at every key: each wave sorts its 64 keys in registers, leaves the sorted run in the LDS, and a
// key's rank is its place in its own run plus, by bisection, the keys below it in every other run (7 probes per
// run where counting took one read and one compare per worker).  The carry is WideCarry's, the key in its low word.
constexpr uint32_t W32_FULL = ~(uint32_t)WIDE_ID_MASK;               // | worker id: full (or absent) worker
constexpr uint32_t W32_ID_MASK = (uint32_t)WIDE_ID_MASK;
static_assert(((uint64_t)PACKED_MAX_LEN << WIDE_ID_BITS) < (1ull << 27), "a round adds less than 2^27 to a key");

// Keys of run r (64 ascending words) below v, for four runs at a time (their probes do not depend on each other).
__device__ __forceinline__ int keys_below4(const uint32_t* run, const int (&r)[4], const bool (&use)[4], uint32_t v) {
    int lo[4] = {0, 0, 0, 0};
#pragma unroll
    for (int step = WAVE / 2; step >= 1; step >>= 1) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (run[r[i] * WAVE + lo[i] + step - 1] < v) lo[i] += step;
    }
    int below = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (run[r[i] * WAVE + lo[i]] < v) lo[i] += 1;                 // (all 64 below)
        below += use[i] ? lo[i] : 0;
    }
    return below;
}

__device__ __forceinline__ int lpt_rounds_wide32_portion(BalLds& L, int N, int P, int C, const uint16_t* sorted,
                                                         uint16_t* step_slot, WideCarry& carry) {
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    const int nw = (P + WAVE - 1) / WAVE;                             // waves that keep workers
    uint32_t* run = reinterpret_cast<uint32_t*>(L.cnt);               // every wave's keys, sorted
    uint32_t* sbuf = run + DC_MAX_SHARDS;                             // keys in rank order
    uint32_t* kbuf = sbuf + DC_MAX_SHARDS;                            // the updated keys on their way back to the workers
    static_assert(3 * DC_MAX_SHARDS <= 256 * BAL_WAVES, "three key tables fit the counters");
    const uint32_t full = W32_FULL | (uint32_t)tid;
    uint32_t key = carry.key >= WIDE_FULL ? full : (uint32_t)carry.key;
    int32_t count = carry.count;
    int64_t load = carry.load;
    int pos = 0;
    uint32_t low = 0;                                                 // the smallest key of the round before (uniform)
    while (pos < N) {                                                 // pos is the same in every thread
        if (low >= 0x40000000u && low < W32_FULL && key < W32_FULL) key -= low & ~W32_ID_MASK;      // rebase
        uint32_t mine = 0xFFFFFFFFu;                                  // lane r of wave w: the r-th smallest key of the wave
        if (w < nw) {                                                 // (uniform)
            mine = wave_sort_asc<WAVE>(key);
            run[tid] = mine;
        }
        __syncthreads();
        if (w < nw) {
            int rank = lane;
            for (int q0 = 0; q0 < nw; q0 += 4) {                      // (uniform)
                int r[4];
                bool use[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    use[i] = q0 + i < nw && q0 + i != w;
                    r[i] = min(q0 + i, nw - 1);
                }
                rank += keys_below4(run, r, use, mine);
            }
            sbuf[min(rank, DC_MAX_SHARDS - 1)] = mine;                // (keys are distinct: every rank is taken once)
        }
        __syncthreads();
        // ---- rank view: thread r offers item I[pos + r] to the worker with the r-th smallest key ----
        const uint32_t sk = tid < P ? sbuf[tid] : 0xFFFFFFFFu;
        low = sbuf[0];
        const int t = pos + tid;
        const bool valid = tid < P && sk < W32_FULL && t < N;
        const uint32_t s = valid ? (uint32_t)L.keys[sorted[t]] : 0u;
        const uint32_t newk = valid ? sk + (s << WIDE_ID_BITS) : 0xFFFFFFFFu;
        // smallest updated key among the ranks below mine
        const uint32_t inc = wave_incl_scan_umin(newk);
        uint32_t pm = dpp_mov<DPP_WAVE_SHR1>(0xFFFFFFFFu, inc);
        if (lane == WAVE - 1) L.tmp32[w] = inc;
        __syncthreads();
        for (int q = 0; q < w; ++q) pm = umin32(pm, L.tmp32[q]);
        // accepted prefix: ranks below the first one whose worker is no longer the minimum
        const uint64_t fail = __ballot(!(valid && sk < pm));
        if (lane == 0) L.red[w] = fail ? w * WAVE + (__ffsll((long long)fail) - 1) : BAL_BLOCK;
        __syncthreads();
        int m = BAL_BLOCK;
        for (int q = 0; q < BAL_WAVES; ++q) m = min(m, L.red[q]);
        if (m == 0) break;                                            // cannot happen: cap * P >= N (uniform)
        // back to the workers: rank r sends its updated key, its own rank in place of the worker id
        if (tid < m) kbuf[sk & W32_ID_MASK] = (newk & ~W32_ID_MASK) | (uint32_t)tid;
        const uint32_t thr = sbuf[m - 1];
        __syncthreads();
        if (tid < P && key <= thr) {                                  // my worker is among the m smallest
            const uint32_t recv = kbuf[tid];
            const uint32_t nk = (recv & ~W32_ID_MASK) | (uint32_t)tid;
            const int took = pos + (int)(recv & W32_ID_MASK);         // the item I took
            step_slot[took] = (uint16_t)count;
            L.keys[sorted[took]] = tid;                               // placed: its length is not needed again
            load += (int64_t)((nk - key) >> WIDE_ID_BITS);
            count += 1;
            key = (count == C) ? full : nk;
        }
        pos += m;
        // (the next round writes run[] first; sbuf and kbuf are rewritten two and four barriers from here)
    }
    carry.key = key >= W32_FULL ? (WIDE_FULL | (uint64_t)tid) : (uint64_t)key;
    carry.count = count; carry.load = load;
    return pos;
}

// After the last portion: part_off[0..P] gets the start of every P_k, the outputs their tables (N: all items).
__device__ __forceinline__ void lpt_wide_finish(BalLds& L, int N, int P, const WideCarry& carry,
                                                int32_t* __restrict__ shard_seq_off, int64_t* __restrict__ shard_load) {
    const int tid = threadIdx.x;
    __syncthreads();                                                  // kbuf / sbuf are done with: the tables take their place
    int32_t total;
    const int32_t off = block_excl_scan_add<int32_t>(carry.count, reinterpret_cast<int32_t*>(L.tmp32), &total);
    int32_t* part_off = reinterpret_cast<int32_t*>(L.cnt) + PART_OFF_AT;
    if (tid < P) { part_off[tid] = off; shard_seq_off[tid] = off; shard_load[tid] = carry.load; }
    if (tid == 0) { part_off[P] = total; shard_seq_off[P] = N; }
}

__device__ __forceinline__ int lpt_rounds_wide(BalLds& L, int N, int P, int C, const uint16_t* sorted, uint16_t* step_slot,
                                               int32_t max_len, int32_t* __restrict__ shard_seq_off,
                                               int64_t* __restrict__ shard_load) {
    WideCarry carry = wide_fresh(P, C);
    const int placed = (uint32_t)max_len <= PACKED_MAX_LEN ? lpt_rounds_wide32_portion(L, N, P, C, sorted, step_slot, carry)
                                                           : lpt_rounds_wide_portion(L, N, P, C, sorted, step_slot, carry);
    lpt_wide_finish(L, N, P, carry, shard_seq_off, shard_load);
    return placed;
}

// The whole of Algorithm 1, by one workgroup of BAL_BLOCK threads.
// What a lane hands to the plan when that runs as the tail of this workgroup: the sequence and the length of
// output slots tid, tid + BAL_BLOCK, ... (seq = -1, len = 0 beyond N).
struct SlotRegs {
    int32_t seq[BAL_ROUNDS];
    int32_t len[BAL_ROUNDS];
};

// FILL (only with P <= 32 or P == 64, and P * C == N): also fill slots; the code of other shapes is left out (the
// kernel is executed once from front to back, most of it straight code that the instruction cache has not seen,
// and its size shows in its time).
template <bool FILL>
__device__ __forceinline__ void balance_body_t(BalLds& L, int32_t N, int32_t P, int32_t C,
                                               const int32_t* __restrict__ seq_len, int32_t* __restrict__ perm,
                                               int32_t* __restrict__ shard_seq_off, int32_t* __restrict__ shard_of_seq,
                                               int64_t* __restrict__ shard_load, int32_t* status, SlotRegs& slots) {
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;

    // every partition ends with exactly C items (Algorithm 1 as printed: C = N / K): rows per worker
    const int pitch = (P <= WAVE && C > 0 && (int64_t)P * C == N) ? place_pitch(C) : 0;
    const bool tight = pitch != 0 && (P <= 32 || P == 64);                  // what the packed rounds serve
    const bool exact = pitch != 0 && (P == 16 || P == 32 || P == 64);      // a worker in every lane of a 16-, 32- or 64-lane sort
    if (tight) bin_sort_clear(L);                                 // (uniform; the barrier below stands between this and the bins' use)

    // ---- load lengths, range (register q of a thread: sequence bal_item(q, rounds)) ----
    const int rounds = (N + BAL_BLOCK - 1) / BAL_BLOCK;           // <= BAL_ROUNDS
    int32_t mx = 0, mn = INT32_MAX;
    int32_t mine_len[BAL_ROUNDS];
#pragma unroll
    for (int q = 0; q < BAL_ROUNDS; ++q) {
        const int i = bal_item(q, rounds);
        mine_len[q] = 1;
        if (q < rounds && i < N) {
            int32_t s = seq_len[i];
            if (s <= 0 || s > DC_MAX_SEQ_LEN) { set_status(status, DC_ERR_ZERO_LENGTH_SEQ); s = 1; }
            mine_len[q] = s;
            mx = max(mx, s);
            mn = min(mn, s);
        }
    }
    wave_all_reduce([&](auto j) {                                 // (lengths are positive: unsigned order is theirs)
        constexpr int J = decltype(j)::value;
        const uint32_t hi = lane_xor<J>((uint32_t)mx), lo = lane_xor<J>((uint32_t)mn);
        mx = max(mx, (int32_t)hi);
        mn = min(mn, (int32_t)lo);
    });
    if (lane == 0) { L.red[w] = mx; L.red[BAL_WAVES + w] = mn; }
    __syncthreads();
    mx = 0; mn = INT32_MAX;
    for (int i = 0; i < BAL_WAVES; ++i) { mx = max(mx, L.red[i]); mn = min(mn, L.red[BAL_WAVES + i]); }
    const uint32_t range = N > 0 ? (uint32_t)(mx - mn) : 0u;
    const int nbits = 32 - __clz(range | 1u);
    const int passes = range == 0 ? 0 : (nbits + 7) / 8;
    int32_t* part_off = reinterpret_cast<int32_t*>(L.cnt) + PART_OFF_AT;
    int32_t* placed = reinterpret_cast<int32_t*>(L.cnt) + PLACED_AT;

    // ---- the printed algorithm on up to 32 or on 64 workers with lengths below 2^16 (lpt_rounds_packed) ----
    // One word per sequence, length << 16 | index, is all that is kept: the sort moves those words between
    // the two halves of the LDS (a pass takes its digit from the word it moves, not from a table of lengths),
    // the rounds read them in sorted order, and the half the sort ends in leaves the other one to the workers'
    // rows.
    if (tight && (uint32_t)mx <= PACKED_MAX_LEN) {                // (uniform)
        static_assert(offsetof(BalLds, idx_b) == offsetof(BalLds, idx_a) + sizeof(uint16_t) * (DC_MAX_SEQ + PLACE_PAD) &&
                      offsetof(BalLds, idx_a) % 4 == 0, "the two index arrays are one run of words");
        uint32_t* src = reinterpret_cast<uint32_t*>(L.keys);      // DC_MAX_SEQ + PLACE_PAD words each
        uint32_t* dst = reinterpret_cast<uint32_t*>(L.idx_a);
        if (range != 0u && range <= BIN_RANGE_MAX && bin_sort_packed(L, N, (uint32_t)mx, range, mine_len, dst)) {     // (uniform)
            uint32_t* t = src; src = dst; dst = t;
        } else {
#pragma unroll
            for (int q = 0; q < BAL_ROUNDS; ++q) {
                const int i = bal_item(q, rounds);
                if (q < rounds && i < N) src[i] = ((uint32_t)mine_len[q] << 16) | (uint32_t)i;
            }
            __syncthreads();
            for (int pass = 0; pass < passes; ++pass) {
                const int shift = pass * 8;
                counting_pass(L, N, rounds,
                              [&](int pos) { return ((uint32_t)mx - (src[pos] >> 16)) >> shift; },
                              [&](int pos, int out) { dst[out] = src[pos]; });
                uint32_t* t = src; src = dst; dst = t;
            }
        }
        uint32_t* const items = src;                              // I of Algorithm 1, each entry with its length
        uint32_t* const rows = dst;
        if (tid < PLACE_PAD) items[N + tid] = 0;                  // the rounds read a little beyond the last item
        __syncthreads();
        const int rpitch = row_pitch(C);
        if (w == 0) {
            int32_t* worker_count = reinterpret_cast<int32_t*>(L.cnt) + WCOUNT_AT;
            uint32_t* spare = reinterpret_cast<uint32_t*>(L.spare);
            int n_placed;
            if (P <= 8) n_placed = lpt_rounds_packed<8>(N, P, C, items, mx, rows, rpitch, spare, worker_count, shard_load);
            else if (P <= 16) n_placed = lpt_rounds_packed<16>(N, P, C, items, mx, rows, rpitch, spare, worker_count, shard_load);
            else if (P <= 32) n_placed = lpt_rounds_packed<32>(N, P, C, items, mx, rows, rpitch, spare, worker_count, shard_load);
            else n_placed = lpt_rounds_packed<64>(N, P, C, items, mx, rows, rpitch, spare, worker_count, shard_load);
            const int32_t c = worker_count[lane];
            const int32_t inc = (int32_t)wave_incl_scan_add_u32((uint32_t)c);
            if (lane < P) shard_seq_off[lane] = inc - c;
            if (lane == 0) { shard_seq_off[P] = N; *placed = n_placed; }
        }
        __syncthreads();
        // ---- P_0, P_1, ... are the rows; the worker of a sequence is the row it stands in ----
        // (gathered by sequence in the LDS, where the sorted items were, so that both outputs leave in index
        // order: 16 384 scattered 4-byte stores take longer to drain than the rounds save)
        uint32_t* const worker_of = items;
        // (slot q = worker q / C, place q mod C: one division per lane, then steps of BAL_BLOCK slots)
        const int step_k = BAL_BLOCK / C, step_r = BAL_BLOCK - step_k * C;
        int k = tid / C, r = tid - k * C;
#pragma unroll
        for (int qq = 0; qq < BAL_ROUNDS; ++qq) {
            const int q = qq * BAL_BLOCK + tid;
            if constexpr (FILL) { slots.seq[qq] = -1; slots.len[qq] = 0; }
            if (q < N) {
                const uint32_t e = rows[k * rpitch + r];
                const uint32_t u = min(e & 0xFFFFu, (uint32_t)(N - 1));      // (no index leaves the arrays whatever a word holds)
                perm[q] = (int32_t)u;
                worker_of[u] = (uint32_t)k;
                if constexpr (FILL) { slots.seq[qq] = (int32_t)u; slots.len[qq] = (int32_t)(e >> 16); }
            }
            k += step_k;
            r += step_r;
            if (r >= C) { r -= C; k += 1; }
        }
        __syncthreads();
        for (int i = tid; i < N; i += BAL_BLOCK) shard_of_seq[i] = (int32_t)worker_of[i];
        return;
    }

#pragma unroll
    for (int q = 0; q < BAL_ROUNDS; ++q) {
        const int i = bal_item(q, rounds);
        if (q < rounds && i < N) L.keys[i] = mine_len[q];
    }
    // ---- a) radix sort of indices by (mx - len) ascending, stable ----
    for (int i = tid; i < N; i += BAL_BLOCK) L.idx_a[i] = (uint16_t)i;
    uint16_t* src = L.idx_a;
    uint16_t* dst = L.idx_b;
    __syncthreads();
    for (int pass = 0; pass < passes; ++pass) {
        const int shift = pass * 8;
        counting_pass(L, N, rounds,
                      [&](int pos) { return ((uint32_t)(mx - L.keys[src[pos]])) >> shift; },
                      [&](int pos, int out) { dst[out] = src[pos]; });
        uint16_t* t = src; src = dst; dst = t;
    }
    const uint16_t* sorted = src;                                 // I of Algorithm 1
    uint16_t* step_slot = dst;                                    // place of I[t] inside its worker's partition
    // ---- b) assignment rounds: wave 0 for up to 64 workers, else the whole workgroup ----
    // (FILL: the caller has up to 32 or 64 workers and equal partitions; the other shapes' code stays out of its kernel)
    if (!FILL && P > WAVE) {
        if constexpr (!FILL) {
            const int n_placed = lpt_rounds_wide(L, N, P, C, sorted, step_slot, mx, shard_seq_off, shard_load);
            if (tid == 0) *placed = n_placed;
        }
    } else if (w == 0) {
        int32_t* worker_count = reinterpret_cast<int32_t*>(L.cnt) + WCOUNT_AT;
        int32_t* spare = L.spare;
        LptCarry fresh = lpt_fresh(P, C);
        int n_placed = 0;
        if (exact && P == 16) n_placed = lpt_rounds<16, true>(N, P, C, L.keys, sorted, mx, step_slot, pitch, spare, worker_count, shard_load, fresh);
        else if (exact && P == 32) n_placed = lpt_rounds<32, true>(N, P, C, L.keys, sorted, mx, step_slot, pitch, spare, worker_count, shard_load, fresh);
        else if (exact) n_placed = lpt_rounds<64, true>(N, P, C, L.keys, sorted, mx, step_slot, pitch, spare, worker_count, shard_load, fresh);
        else if (P <= 16) n_placed = lpt_rounds<16>(N, P, C, L.keys, sorted, mx, step_slot, pitch, spare, worker_count, shard_load, fresh);
        else if (P <= 32) n_placed = lpt_rounds<32>(N, P, C, L.keys, sorted, mx, step_slot, pitch, spare, worker_count, shard_load, fresh);
        else if constexpr (!FILL) n_placed = lpt_rounds<64>(N, P, C, L.keys, sorted, mx, step_slot, pitch, spare, worker_count, shard_load, fresh);
        // start of every P_k inside perm
        const int32_t c = worker_count[lane];
        const int32_t inc = (int32_t)wave_incl_scan_add_u32((uint32_t)c);
        part_off[lane] = inc - c;
        if (lane < P) shard_seq_off[lane] = inc - c;
        if (lane == 0) { shard_seq_off[P] = N; *placed = n_placed; }
    }
    __syncthreads();

    // ---- c) lay out P_0, P_1, ... each in insertion order ----
    const int n_placed = *placed;
    if (pitch) {                                                  // both stores in index order
        const int step_k = BAL_BLOCK / C, step_r = BAL_BLOCK - step_k * C;
        int k = tid / C, r = tid - k * C;                         // slot q = worker q / C, place q mod C
#pragma unroll
        for (int qq = 0; qq < BAL_ROUNDS; ++qq) {
            const int q = qq * BAL_BLOCK + tid;
            if constexpr (FILL) { slots.seq[qq] = -1; slots.len[qq] = 0; }
            if (q < N) {
                const int u = min((int)step_slot[k * pitch + r], N - 1);
                perm[q] = u;
                shard_of_seq[q] = L.keys[q];
                if constexpr (FILL) {                             // (lengths of 2^16 and more: they are in global memory only)
                    const int32_t s = seq_len[u];
                    slots.seq[qq] = u;
                    slots.len[qq] = (s <= 0 || s > DC_MAX_SEQ_LEN) ? 1 : s;
                }
            }
            k += step_k;
            r += step_r;
            if (r >= C) { r -= C; k += 1; }
        }
        return;
    }
    for (int t = tid; t < n_placed; t += BAL_BLOCK) {
        const int u = sorted[t];
        const int k = L.keys[u];                                  // the worker that took it
        shard_of_seq[u] = k;
        perm[part_off[k] + step_slot[t]] = u;
    }
}

__device__ __forceinline__ void balance_body(BalLds& L, int32_t N, int32_t P, int32_t C,
                                             const int32_t* __restrict__ seq_len, int32_t* __restrict__ perm,
                                             int32_t* __restrict__ shard_seq_off, int32_t* __restrict__ shard_of_seq,
                                             int64_t* __restrict__ shard_load, int32_t* status) {
    SlotRegs unused;
    balance_body_t<false>(L, N, P, C, seq_len, perm, shard_seq_off, shard_of_seq, shard_load, status, unused);
}

}  // namespace dc
