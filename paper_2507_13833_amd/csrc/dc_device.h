// Device-side building blocks shared by the reshard kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "dc_internal.h"

namespace dc {

constexpr int WAVE = 64;

// First device-side error wins.
__device__ __forceinline__ void set_status(int32_t* d_status, int32_t code) {
    if (d_status) atomicCAS(d_status, 0, code);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (WAVE - 1); }

// ---- wave64 scans: six steps of register moves between lanes (DPP), nothing goes through the LDS unit ----
// Step controls: lane i takes lane i - 1 / 2 / 4 / 8 of its row of 16; then lane 15 of a row is sent to every lane of
// the next row (rows 1 and 3), then lane 31 to rows 2 and 3.  A lane that the step does not reach keeps `identity`.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t scan_step(uint32_t identity, uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, CTRL, ROW_MASK, 0xF, false);
}
template <typename Combine>
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v, uint32_t identity, Combine combine) {
    v = combine(v, scan_step<0x111>(identity, v));
    v = combine(v, scan_step<0x112>(identity, v));
    v = combine(v, scan_step<0x114>(identity, v));
    v = combine(v, scan_step<0x118>(identity, v));
    v = combine(v, scan_step<0x142, 0xA>(identity, v));
    v = combine(v, scan_step<0x143, 0xC>(identity, v));
    return v;
}
__device__ __forceinline__ uint64_t scan_step_add64(uint64_t v, uint32_t lo, uint32_t hi) { return v + (((uint64_t)hi << 32) | lo); }

template <typename T>
__device__ __forceinline__ T wave_incl_scan_add(T v) {
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "32- or 64-bit integers");
    if constexpr (sizeof(T) == 4) {
        return (T)wave_incl_scan_u32((uint32_t)v, 0u, [](uint32_t a, uint32_t b) { return a + b; });
    } else {
        uint64_t x = (uint64_t)v;                         // both halves take the same step; the carry is the adder's
        x = scan_step_add64(x, scan_step<0x111>(0u, (uint32_t)x), scan_step<0x111>(0u, (uint32_t)(x >> 32)));
        x = scan_step_add64(x, scan_step<0x112>(0u, (uint32_t)x), scan_step<0x112>(0u, (uint32_t)(x >> 32)));
        x = scan_step_add64(x, scan_step<0x114>(0u, (uint32_t)x), scan_step<0x114>(0u, (uint32_t)(x >> 32)));
        x = scan_step_add64(x, scan_step<0x118>(0u, (uint32_t)x), scan_step<0x118>(0u, (uint32_t)(x >> 32)));
        x = scan_step_add64(x, scan_step<0x142, 0xA>(0u, (uint32_t)x), scan_step<0x142, 0xA>(0u, (uint32_t)(x >> 32)));
        x = scan_step_add64(x, scan_step<0x143, 0xC>(0u, (uint32_t)x), scan_step<0x143, 0xC>(0u, (uint32_t)(x >> 32)));
        return (T)x;
    }
}

__device__ __forceinline__ int32_t wave_incl_scan_max(int32_t v) {
    return (int32_t)wave_incl_scan_u32((uint32_t)v, (uint32_t)INT32_MIN,
                                       [](uint32_t a, uint32_t b) { return (uint32_t)max((int32_t)a, (int32_t)b); });
}
// The value of the lane before (lane 0: `first`).
__device__ __forceinline__ int32_t wave_shift_up1(int32_t v, int32_t first) {
    return (int32_t)scan_step<0x138>((uint32_t)first, (uint32_t)v);
}

// The value that lane `from` (the same in every lane of the wave) holds.
template <typename T>
__device__ __forceinline__ T wave_read_lane(T v, int from) {
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "32- or 64-bit integers");
    const int at = __builtin_amdgcn_readfirstlane(from);
    if constexpr (sizeof(T) == 4) {
        return (T)__builtin_amdgcn_readlane((int)v, at);
    } else {
        const uint64_t x = (uint64_t)v;
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, at);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), at);
        return (T)(((uint64_t)hi << 32) | lo);
    }
}

// Block-wide exclusive add-scan of one value per thread.  `tmp` holds one T per
// wave (at most 64).  Returns the exclusive prefix; *total gets the block sum.
// Contains __syncthreads(): every thread of the block must call it.
// (The waves' sums are scanned by every wave for itself, lane i taking wave i's: one LDS read and a register
// scan, where a loop over the waves would wait for the LDS once per wave.)
template <typename T>
__device__ __forceinline__ T block_excl_scan_add(T v, T* tmp, T* total) {
    const int lane = lane_id(), w = threadIdx.x / WAVE, nw = blockDim.x / WAVE;
    T inc = wave_incl_scan_add(v);
    if (lane == WAVE - 1) tmp[w] = inc;
    __syncthreads();
    const T mine = lane < nw ? tmp[lane] : T(0);
    const T upto = wave_incl_scan_add(mine);
    __syncthreads();
    *total = wave_read_lane(upto, WAVE - 1);
    return wave_read_lane((T)(upto - mine), w) + inc - v;
}

// Block-wide exclusive max-scan (identity -1).
__device__ __forceinline__ int32_t block_excl_scan_max(int32_t v, int32_t* tmp) {
    const int lane = lane_id(), w = threadIdx.x / WAVE, nw = blockDim.x / WAVE;
    int32_t inc = wave_incl_scan_max(v);
    if (lane == WAVE - 1) tmp[w] = inc;
    __syncthreads();
    const int32_t upto = wave_incl_scan_max(lane < nw ? tmp[lane] : -1);
    const int32_t base = wave_read_lane(wave_shift_up1(upto, -1), w);
    const int32_t up = wave_shift_up1(inc, -1);
    __syncthreads();
    return max(base, up);
}

// ---- 16-byte global accesses ----
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));

// 16 bytes from a 4-byte aligned address, streamed (no reuse expected).
__device__ __forceinline__ u32x4 load16_a4(const void* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_a4*>(p));
}
__device__ __forceinline__ uint32_t load4(const void* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(p));
}
// 16 bytes to a 16-byte aligned address, streamed.
__device__ __forceinline__ void store16(void* p, u32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
}

}  // namespace dc
