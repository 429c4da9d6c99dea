// Algorithm 1, Constrained LPT Load Balancing (Sec. 6 "Load Balancing").
//
// One workgroup, everything in LDS (N <= DC_MAX_SEQ, P <= DC_MAX_SHARDS):
//   a) stable LSD radix sort of the sequence indices by descending length
//      (8-bit digits of max_len - len, only as many passes as the length range
//      needs; ranks inside a wave by ballot matching, across waves by a scan of
//      per-wave digit counters);
//   b) the assignment on wave 0, lane k = worker k, in ROUNDS instead of one item
//      per step.  A lane holds its worker's item count and a 32-bit key
//      (load - base) << 6 | k (all-ones-ish when the worker is full).  A round
//      sorts the 64 keys across lanes (bitonic network in DPP), hands the next
//      items, in order, to the workers in key order, and accepts the longest
//      prefix for which "worker of rank j is still the minimum after ranks < j took
//      their items" holds - exactly the sequence of pop_min results Algorithm 1
//      would produce, since rank j is popped next iff its key is below every
//      updated key.  With descending lengths nearly every round places one item
//      on every open worker, so N/P rounds replace N dependent steps.
//      Loads of open workers never differ by more than the longest sequence, so
//      rebasing the keys when the minimum grows keeps them in 32 bits for any
//      total load (the minimum grows by at most one longest sequence per round, so
//      the check runs every so many rounds, not in each);
//      With more than 64 workers the same rounds run on the whole workgroup, thread k = worker
//      k, 64-bit keys load << 10 | k: every thread ranks its key by counting the smaller ones,
//      the accepted prefix comes from a workgroup-wide min-scan, and keys travel between rank
//      order and worker order through LDS;
//   c) a worker that takes an item notes the item's place inside P_k (its item count before) and
//      its own id (in LDS, where the item's length was); when all items are placed, a scan of the
//      workers' counts gives the start of every P_k and one pass writes perm (P_0, P_1, ... each in
//      insertion order) and the worker of every sequence.  When N = P * C (the algorithm as printed)
//      every P_k ends with C items, the items are filed per worker as they are placed, and both
//      outputs are written in index order.
#include "balance_device.h"
#include "plan_device.h"

namespace dc {

__global__ __launch_bounds__(BAL_BLOCK) void balance_kernel(int32_t N, int32_t P, int32_t C,
                                                            const int32_t* __restrict__ seq_len,
                                                            int32_t* __restrict__ perm,
                                                            int32_t* __restrict__ shard_seq_off,
                                                            int32_t* __restrict__ shard_of_seq,
                                                            int64_t* __restrict__ shard_load,
                                                            int32_t* status) {
    __shared__ BalLds L;
    balance_body(L, N, P, C, seq_len, perm, shard_seq_off, shard_of_seq, shard_load, status);
}

// Balance and the group-relative advantage in ONE launch: workgroup 0 is the balance workgroup, every
// other workgroup gives its 16 waves to 16 sequences of the advantage stage.  The two stages are
// independent and the balance occupies one compute unit for its whole (latency-bound) run, so the
// advantage stage's HBM traffic hides behind it - without a second stream and the two cross-stream
// waits per step that go with it (several microseconds each).  The advantage workgroups carry the
// balance workgroup's LDS allocation, i.e. one of them fits a compute unit: half the waves the
// stage has as a kernel of its own, still well inside the balance's run time.
struct BalanceArgs {
    int32_t N, P, C;
    const int32_t* seq_len;
    int32_t* perm;
    int32_t* shard_seq_off;
    int32_t* shard_of_seq;
    int64_t* shard_load;
    int32_t* status;
};

__global__ __launch_bounds__(BAL_BLOCK) void balance_advantage_kernel(BalanceArgs b, AdvArgs a, SourceDesc sd) {
    __shared__ BalLds L;
    if (blockIdx.x == 0)
        balance_body(L, b.N, b.P, b.C, b.seq_len, b.perm, b.shard_seq_off, b.shard_of_seq, b.shard_load, b.status);
    else
        advantage_wave(a, sd, (int64_t)(blockIdx.x - 1) * BAL_WAVES + __builtin_amdgcn_readfirstlane((int)(threadIdx.x / WAVE)));
}

// The same launch with the plan of the packed training layout as the tail of the balance workgroup: when
// Algorithm 1 is done the workgroup holds every output slot's sequence and length, which is all the plan
// reads, so the plan's own launch, the gathers of lengths through perm in front of it (slots_kernel) and
// its permutation check fall away.  The LDS is Algorithm 1's first and the plan's afterwards.
static_assert(BAL_BLOCK == PLAN_BLOCK && BAL_ROUNDS == PLAN_IPT, "one lane handles the same slots in both");
constexpr size_t BAL_PLAN_LDS = sizeof(BalLds) > sizeof(PlanLds) ? sizeof(BalLds) : sizeof(PlanLds);

__global__ __launch_bounds__(BAL_BLOCK) void balance_plan_advantage_kernel(BalanceArgs b, PlanArgs p, AdvArgs a, SourceDesc sd) {
    __shared__ __align__(16) unsigned char lds[BAL_PLAN_LDS];
    if (blockIdx.x != 0) {
        advantage_wave(a, sd, (int64_t)(blockIdx.x - 1) * BAL_WAVES + __builtin_amdgcn_readfirstlane((int)(threadIdx.x / WAVE)));
        return;
    }
    SlotRegs s;
    balance_body_t<true>(*reinterpret_cast<BalLds*>(lds), b.N, b.P, b.C, b.seq_len, b.perm, b.shard_seq_off, b.shard_of_seq,
                         b.shard_load, b.status, s);
#pragma unroll
    for (int q = 0; q < PLAN_IPT; ++q) {                          // the slots' lengths, for the launch that builds the granule tables
        const int j = q * PLAN_BLOCK + (int)threadIdx.x;
        if (j < b.N) p.slot_len[j] = s.len[q];
    }
    __syncthreads();                                              // Algorithm 1's tables have been read for the last time
    plan_body(*reinterpret_cast<PlanLds*>(lds), p, s.seq, s.len, false, b.C);
}

hipError_t launch_balance(int32_t n_seq, int32_t n_shards, int32_t cap_eff, const int32_t* d_seq_len,
                          int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                          int64_t* d_shard_load, int32_t* d_status, hipStream_t st) {
    hipLaunchKernelGGL(balance_kernel, dim3(1), dim3(BAL_BLOCK), 0, st, n_seq, n_shards, cap_eff, d_seq_len,
                       d_perm, d_shard_seq_off, d_shard_of_seq, d_shard_load, d_status);
    return hipGetLastError();
}

hipError_t launch_balance_advantage(int32_t n_seq, int32_t n_shards, int32_t cap_eff, const int32_t* d_seq_len,
                                    int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                                    int64_t* d_shard_load, const AdvArgs& adv, const SourceDesc& src,
                                    int32_t n_groups, int32_t* d_status, hipStream_t st) {
    BalanceArgs b;
    b.N = n_seq; b.P = n_shards; b.C = cap_eff; b.seq_len = d_seq_len; b.perm = d_perm;
    b.shard_seq_off = d_shard_seq_off; b.shard_of_seq = d_shard_of_seq; b.shard_load = d_shard_load; b.status = d_status;
    const int64_t grid = 1 + (adv_waves(n_seq, n_groups) + BAL_WAVES - 1) / BAL_WAVES;
    hipLaunchKernelGGL(balance_advantage_kernel, dim3((unsigned)grid), dim3(BAL_BLOCK), 0, st, b, adv, src);
    return hipGetLastError();
}

hipError_t launch_balance_plan_advantage(int32_t n_seq, int32_t n_shards, int32_t cap_eff, const int32_t* d_seq_len,
                                         int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                                         int64_t* d_shard_load, const PlanArgs& plan, const AdvArgs& adv,
                                         const SourceDesc& src, int32_t n_groups, int32_t* d_status, hipStream_t st) {
    // (the kernel holds the code of these shapes only)
    if (!((n_shards >= 1 && n_shards <= 32) || n_shards == 64) || (int64_t)cap_eff * n_shards != n_seq || n_seq <= 0 || n_seq > DC_MAX_SEQ)
        return hipErrorInvalidValue;
    BalanceArgs b;
    b.N = n_seq; b.P = n_shards; b.C = cap_eff; b.seq_len = d_seq_len; b.perm = d_perm;
    b.shard_seq_off = d_shard_seq_off; b.shard_of_seq = d_shard_of_seq; b.shard_load = d_shard_load; b.status = d_status;
    const int64_t grid = 1 + (adv_waves(n_seq, n_groups) + BAL_WAVES - 1) / BAL_WAVES;
    hipLaunchKernelGGL(balance_plan_advantage_kernel, dim3((unsigned)grid), dim3(BAL_BLOCK), 0, st, b, plan, adv, src);
    return hipGetLastError();
}

}  // namespace dc
