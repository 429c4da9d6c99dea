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

// ---- wave64 scans (shuffles lower to DPP / ds_bpermute) ----
template <typename T>
__device__ __forceinline__ T wave_incl_scan_add(T v) {
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {
        T o = __shfl_up(v, d, WAVE);
        if (lane >= d) v += o;
    }
    return v;
}

__device__ __forceinline__ int32_t wave_incl_scan_max(int32_t v) {
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {
        int32_t o = __shfl_up(v, d, WAVE);
        if (lane >= d) v = max(v, o);
    }
    return v;
}

// Block-wide exclusive add-scan of one value per thread.  `tmp` holds one T per
// wave (at most 16).  Returns the exclusive prefix; *total gets the block sum.
// Contains __syncthreads(): every thread of the block must call it.
template <typename T>
__device__ __forceinline__ T block_excl_scan_add(T v, T* tmp, T* total) {
    const int lane = lane_id(), w = threadIdx.x / WAVE, nw = blockDim.x / WAVE;
    T inc = wave_incl_scan_add(v);
    if (lane == WAVE - 1) tmp[w] = inc;
    __syncthreads();
    T base = 0, sum = 0;
    for (int i = 0; i < nw; ++i) {
        T x = tmp[i];
        if (i < w) base += x;
        sum += x;
    }
    __syncthreads();
    *total = sum;
    return base + inc - v;
}

// Block-wide exclusive max-scan (identity -1).
__device__ __forceinline__ int32_t block_excl_scan_max(int32_t v, int32_t* tmp) {
    const int lane = lane_id(), w = threadIdx.x / WAVE;
    int32_t inc = wave_incl_scan_max(v);
    if (lane == WAVE - 1) tmp[w] = inc;
    __syncthreads();
    int32_t base = -1;
    for (int i = 0; i < w; ++i) base = max(base, tmp[i]);
    int32_t up = __shfl_up(inc, 1, WAVE);
    if (lane == 0) up = -1;
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
