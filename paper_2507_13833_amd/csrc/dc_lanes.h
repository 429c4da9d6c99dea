// Cross-lane primitives for wave64 on gfx950: partner exchange lane ^ J, a 64-lane
// bitonic sort of unsigned keys, and min scans.  All data stays in VGPRs (DPP,
// v_permlane*_swap); nothing touches LDS memory.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace dc {

// DPP controls
constexpr int DPP_QUAD_PERM_1032 = 0xB1;    // lane ^ 1
constexpr int DPP_QUAD_PERM_2301 = 0x4E;    // lane ^ 2
constexpr int DPP_ROW_SHL4 = 0x104;         // lane i <- lane i+4 (within a row of 16)
constexpr int DPP_ROW_SHR1 = 0x111;         // lane i <- lane i-1
constexpr int DPP_ROW_SHR2 = 0x112;
constexpr int DPP_ROW_SHR4 = 0x114;
constexpr int DPP_ROW_SHR8 = 0x118;
constexpr int DPP_ROW_ROR8 = 0x128;         // lane ^ 8
constexpr int DPP_WAVE_SHR1 = 0x138;        // lane i <- lane i-1 across the whole wave
constexpr int DPP_ROW_BCAST15 = 0x142;      // lane 15 of each row -> every lane of the next row
constexpr int DPP_ROW_BCAST31 = 0x143;      // lane 31 -> every lane of rows 2 and 3

template <int CTRL, int ROW_MASK = 0xF, int BANK_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t old, uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)v, CTRL, ROW_MASK, BANK_MASK, false);
}
// Every lane is written (full row and bank masks, every source lane exists): no previous value to keep.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_perm(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xF, 0xF, false);
}

// The same with one more (unused) scalar operand: the statement cannot be scheduled before `after`
// exists, which places whatever computes `after` in front of it (see wave_sort_asc_tied).
__device__ __forceinline__ uint32_t umed3_after(uint32_t a, uint32_t b, uint32_t c, uint32_t after);

// Median of three unsigned values in one instruction.  med3(a, b, 0) = min(a, b) and
// med3(a, b, ~0) = max(a, b), so a per-lane constant chooses between the two.  (The compiler
// treats the statement's output like any vector-ALU result and keeps the idle cycles a DPP
// read of it needs.)
__device__ __forceinline__ uint32_t umed3(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t r;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

__device__ __forceinline__ uint32_t umed3_after(uint32_t a, uint32_t b, uint32_t c, uint32_t after) {
    uint32_t r;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c), "s"(after));
    return r;
}

// Value of lane (lane ^ J).
template <int J>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v) {
    static_assert(J == 1 || J == 2 || J == 4 || J == 8 || J == 16 || J == 32, "power of two below 64");
    if constexpr (J == 1) return dpp_perm<DPP_QUAD_PERM_1032>(v);
    else if constexpr (J == 2) return dpp_perm<DPP_QUAD_PERM_2301>(v);
    else if constexpr (J == 4) {
        // lanes with bit 2 clear (banks 0, 2) take lane+4, the others lane-4; what the first move leaves in
        // banks 1, 3 does not matter (the second overwrites it), so it needs no previous value and no copy
        uint32_t t = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, DPP_ROW_SHL4, 0xF, 0x5, false);
        return dpp_mov<DPP_ROW_SHR4, 0xF, 0xA>(t, v);
    } else if constexpr (J == 8) return dpp_perm<DPP_ROW_ROR8>(v);
    else if constexpr (J == 16) {
        // swap: a = [r0 r0 r2 r2], b = [r1 r1 r3 r3]; even rows want b, odd rows want a
        auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
        return (threadIdx.x & 16) ? r[0] : r[1];
    } else {
        auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        return (threadIdx.x & 32) ? r[0] : r[1];
    }
}

// step(integral_constant J) for J = 1, 2, 4, 8, 16, 32: the six levels of a butterfly over the 64 lanes.  A step that
// combines every value it keeps with lane_xor<J> of it leaves the reduction over all lanes in every lane.
template <typename Step>
__device__ __forceinline__ void wave_all_reduce(Step step) {
    step(std::integral_constant<int, 1>{});
    step(std::integral_constant<int, 2>{});
    step(std::integral_constant<int, 4>{});
    step(std::integral_constant<int, 8>{});
    step(std::integral_constant<int, 16>{});
    step(std::integral_constant<int, 32>{});
}

template <int K, int J, bool TIED = false>
__device__ __forceinline__ uint32_t bitonic_step(uint32_t v, uint32_t after = 0) {
    const uint32_t lane = threadIdx.x & 63u;
    const bool lower = (lane & J) == 0;          // I am the lower lane of the pair
    const bool asc = (lane & K) == 0;            // my block sorts ascending
    // the lower lane of an ascending pair keeps the smaller key, its partner the larger
    const uint32_t pick = lower == asc ? 0u : 0xFFFFFFFFu;
    if constexpr (J >= 16) {
        // a row swap of v with itself leaves {own key, partner's key} in the two results, in an order
        // that depends on the lane; the median does not care which is which
        if constexpr (J == 16) {
            auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
            return TIED ? umed3_after(r[0], r[1], pick, after) : umed3(r[0], r[1], pick);
        } else {
            auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
            return TIED ? umed3_after(r[0], r[1], pick, after) : umed3(r[0], r[1], pick);
        }
    } else {
        return TIED ? umed3_after(v, lane_xor<J>(v), pick, after) : umed3(v, lane_xor<J>(v), pick);
    }
}

template <int K, int J>
__device__ __forceinline__ uint32_t bitonic_merge(uint32_t v) {
    v = bitonic_step<K, J>(v);
    if constexpr (J > 1) v = bitonic_merge<K, J / 2>(v);
    return v;
}

template <int K, int WIDTH>
__device__ __forceinline__ uint32_t bitonic_sort_levels(uint32_t v) {
    v = bitonic_merge<K, K / 2>(v);
    if constexpr (K < WIDTH) v = bitonic_sort_levels<K * 2, WIDTH>(v);
    return v;
}

// Bitonic sort of each aligned group of WIDTH lanes (WIDTH = 16, 32, 64): even groups
// come out ascending (lane r of group 0 ends with the r-th smallest of lanes
// 0..WIDTH-1), odd groups descending.  Keys need not be distinct.
template <int WIDTH>
__device__ __forceinline__ uint32_t wave_sort_asc(uint32_t v) {
    return bitonic_sort_levels<2, WIDTH>(v);
}

// The two halves of wave_sort_asc: every level but the last, then the last level (the merge of the two
// sorted halves of a group), whose first step waits for the scalar `after`.  A single wave issues in
// order and a dependent vector instruction follows its producer only after about 8 cycles, of which the
// issue takes 4: work that does not depend on the sort runs for free between the sort's steps if
// it stands between them in the instruction stream, and `after` is how the caller puts it there.
template <int WIDTH>
__device__ __forceinline__ uint32_t wave_sort_front(uint32_t v) {
    return bitonic_sort_levels<2, WIDTH / 2>(v);
}
template <int WIDTH>
__device__ __forceinline__ uint32_t wave_sort_back(uint32_t v, uint32_t after) {
    v = bitonic_step<WIDTH, WIDTH / 2, true>(v, after);
    return bitonic_merge<WIDTH, WIDTH / 4>(v);
}

// The same network one compare-exchange at a time, so that a caller can place other work between the
// steps.  Step i of the sort of WIDTH lanes is (net_k(i), net_j(i)): merge size and partner distance.
constexpr int net_steps(int width) {
    int n = 0;
    for (int k = 2; k <= width; k <<= 1)
        for (int j = k >> 1; j >= 1; j >>= 1) ++n;
    return n;
}
constexpr int net_k(int i) {
    for (int k = 2;; k <<= 1)
        for (int j = k >> 1; j >= 1; j >>= 1)
            if (i-- == 0) return k;
}
constexpr int net_j(int i) {
    for (int k = 2;; k <<= 1)
        for (int j = k >> 1; j >= 1; j >>= 1)
            if (i-- == 0) return j;
}
struct XchgPair { uint32_t a, b; };       // a lane's key and its partner's, in either order
// First half of a step: fetch the partner's key (the cross-lane move).
template <int J>
__device__ __forceinline__ XchgPair xchg_fetch(uint32_t v) {
    XchgPair x;
    if constexpr (J == 16) {
        auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
        x.a = r[0]; x.b = r[1];
    } else if constexpr (J == 32) {
        auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        x.a = r[0]; x.b = r[1];
    } else {
        x.a = v; x.b = lane_xor<J>(v);
    }
    return x;
}
// Second half: keep the smaller or the larger of the two (see bitonic_step).
template <int K, int J>
__device__ __forceinline__ uint32_t xchg_keep(XchgPair x) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t pick = ((lane & J) == 0) == ((lane & K) == 0) ? 0u : 0xFFFFFFFFu;
    return umed3(x.a, x.b, pick);
}

// Steps [FROM, TO) of the sort of WIDTH lanes.  side(slot) is called twice per step, with the compile-time
// slot numbers 2 i (between the fetch and the keep of step i) and 2 i + 1 (behind the keep); what it does
// there is issued in the idle cycles between the step's two dependent instructions and must not depend
// on the sort.  The scheduler is told to leave that order alone.
template <int WIDTH, int FROM, int TO, typename Side>
__device__ __forceinline__ uint32_t wave_sort_steps(uint32_t v, Side&& side) {
    if constexpr (FROM < TO) {
        constexpr int K = net_k(FROM), J = net_j(FROM);
        const XchgPair x = xchg_fetch<J>(v);
        __builtin_amdgcn_sched_barrier(0);
        side(std::integral_constant<int, 2 * FROM>{});
        __builtin_amdgcn_sched_barrier(0);
        v = xchg_keep<K, J>(x);
        __builtin_amdgcn_sched_barrier(0);
        side(std::integral_constant<int, 2 * FROM + 1>{});
        __builtin_amdgcn_sched_barrier(0);
        return wave_sort_steps<WIDTH, FROM + 1, TO>(v, side);
    } else {
        return v;
    }
}

__device__ __forceinline__ uint32_t umin32(uint32_t a, uint32_t b) { return a < b ? a : b; }

// Inclusive min-scan over the 64 lanes (lane i: min of lanes 0..i).
__device__ __forceinline__ uint32_t wave_incl_scan_umin(uint32_t v) {
    const uint32_t ID = 0xFFFFFFFFu;
    v = umin32(v, dpp_mov<DPP_ROW_SHR1>(ID, v));
    v = umin32(v, dpp_mov<DPP_ROW_SHR2>(ID, v));
    v = umin32(v, dpp_mov<DPP_ROW_SHR4>(ID, v));
    v = umin32(v, dpp_mov<DPP_ROW_SHR8>(ID, v));
    v = umin32(v, dpp_mov<DPP_ROW_BCAST15, 0xA>(ID, v));
    v = umin32(v, dpp_mov<DPP_ROW_BCAST31, 0xC>(ID, v));
    return v;
}

// Inclusive add-scan over the 64 lanes (lane i: sum of lanes 0..i), same DPP ladder.
__device__ __forceinline__ uint32_t wave_incl_scan_add_u32(uint32_t v) {
    v += dpp_mov<DPP_ROW_SHR1>(0u, v);
    v += dpp_mov<DPP_ROW_SHR2>(0u, v);
    v += dpp_mov<DPP_ROW_SHR4>(0u, v);
    v += dpp_mov<DPP_ROW_SHR8>(0u, v);
    v += dpp_mov<DPP_ROW_BCAST15, 0xA>(0u, v);
    v += dpp_mov<DPP_ROW_BCAST31, 0xC>(0u, v);
    return v;
}

// Exclusive min-scan (lane 0 gets all-ones).
__device__ __forceinline__ uint32_t wave_excl_scan_umin(uint32_t v) {
    return dpp_mov<DPP_WAVE_SHR1>(0xFFFFFFFFu, wave_incl_scan_umin(v));
}

}  // namespace dc
