// dc_repack for callers that cannot hand over a workspace they allocated: the plan's workspace
// (per-slot source descriptors and the per-granule tables the gather reads) lives in a device
// array of fixed size that is part of the library's code object.  Everything else is dc_repack:
// same kernels, same checks, same results.
#include <mutex>
#include "dc_internal.h"

namespace {

// Every GPU the library runs on holds its own copy of this array, at its own address, from the
// time the code object is loaded there until the process ends.  In host code the name is only a
// handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[DC_REPACK_NOALLOC_WS_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
void* g_scratch_of[MAX_DEVICES];        // per device, filled at the first call on that device

// Device address of the current device's copy of the array.
dc_status scratch_of_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return DC_ERR_HIP;
    if (dev < 0 || dev >= MAX_DEVICES) return DC_ERR_UNSUPPORTED_SIZE;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_of[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DC_ERR_HIP;
        g_scratch_of[dev] = p;
    }
    *out = g_scratch_of[dev];
    return DC_OK;
}

}  // namespace

extern "C" dc_status dc_repack_noalloc(const dc_params* prm, const dc_source* src, const int32_t* d_seq_len,
                                       const int32_t* d_perm, const int32_t* d_shard_seq_off,
                                       const dc_field* fields, int32_t n_fields, int64_t dst_capacity_tokens,
                                       int64_t* d_dst_tok_off, int64_t* d_shard_tok_off, int32_t* d_shard_mb_off,
                                       int32_t* d_mb_seq_off, int32_t* d_cu_seqlens, int32_t* d_n_mb,
                                       int32_t* d_status, void* hip_stream) {
    if (!prm) return DC_ERR_INVALID_ARG;
    if (dst_capacity_tokens < 0) return DC_ERR_INVALID_ARG;
    // the sizes must fit the array: checked before anything is enqueued
    if (prm->n_seq < 0) return DC_ERR_INVALID_ARG;
    if (prm->n_seq > DC_MAX_SEQ_LARGE) return DC_ERR_UNSUPPORTED_SIZE;
    const size_t need = dc_workspace_bytes(prm, dst_capacity_tokens);
    if (need == 0 || need > (size_t)DC_REPACK_NOALLOC_WS_BYTES) return DC_ERR_UNSUPPORTED_SIZE;
    void* ws = nullptr;
    const dc_status rc = scratch_of_current_device(&ws);
    if (rc != DC_OK) return rc;
    // The plan writes every table entry the gather reads (padding entries included) before the
    // gather's launch on the same stream, so nothing of the previous call's contents is read.
    return dc_repack(prm, src, d_seq_len, d_perm, d_shard_seq_off, fields, n_fields, dst_capacity_tokens,
                     d_dst_tok_off, d_shard_tok_off, d_shard_mb_off, d_mb_seq_off, d_cu_seqlens, d_n_mb,
                     ws, (size_t)DC_REPACK_NOALLOC_WS_BYTES, d_status, hip_stream);
}
