// Host-side declarations shared by the API layer and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include "../../include/dc.h"

namespace dc {

// Tokens of destination space one gather workgroup owns.  Also the granularity
// of the per-tile "first slot" table the plan kernel leaves in the workspace.
constexpr int GATHER_TILE = 2048;
// Tokens of rollout space one advantage workgroup owns.
constexpr int ADV_TILE = 8192;
// Segment descriptors staged in LDS per pass over a tile, plus look-ahead so a
// 16-token chunk that starts in the last owned segment can be finished.
constexpr int SEG_BATCH = 256;
constexpr int SEG_AHEAD = 16;


// Workspace carved by dc_plan for dc_gather: per-slot source descriptors
// (validated, clamped) and the first slot of every destination tile.
struct Workspace {
    int64_t* slot_src_off;   // [N]   element offset of the slot's sequence in its rollout shard
    int32_t* slot_len;       // [N]   tokens to copy (0 if the slot failed validation)
    int32_t* slot_shard;     // [N]   rollout shard of the slot's sequence
    int32_t* tile_first;     // [n_tiles] first slot whose tokens reach into the tile (N if none)
    int64_t  n_tiles;
    size_t   bytes;
};
Workspace carve_workspace(void* base, int32_t n_seq, int64_t dst_capacity_tokens);

struct SourceDesc {                       // by-value kernel argument
    int32_t n_src;
    int32_t seq_off[DC_MAX_SRC_SHARDS + 1];
    int64_t tokens[DC_MAX_SRC_SHARDS];
};

struct FieldDesc {
    char*       dst;
    int32_t     elem_bytes;
    int32_t     pad;
    const char* src[DC_MAX_SRC_SHARDS];
};
struct FieldTable {                       // by-value kernel argument
    int32_t   n_fields;
    int32_t   n_src;
    FieldDesc f[DC_MAX_FIELDS];
};

hipError_t launch_balance(int32_t n_seq, int32_t n_shards, int32_t cap_eff, const int32_t* d_seq_len,
                          int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                          int64_t* d_shard_load, int32_t* d_status, hipStream_t st);

hipError_t launch_advantage(int32_t n_seq, const SourceDesc& src, const int64_t* d_src_tok_off,
                            const int32_t* d_seq_len, const float* d_reward, const int32_t* d_group_off,
                            int32_t n_groups, double eps, int32_t ddof,
                            const uint8_t* const* mask_base, float* d_adv_seq, float* const* adv_tok_base,
                            int32_t* d_status, hipStream_t st);

hipError_t launch_plan(const dc_params& prm, const SourceDesc& src, const int64_t* d_src_tok_off,
                       const int32_t* d_seq_len, const int32_t* d_perm, const int32_t* d_shard_seq_off,
                       int64_t dst_capacity, int64_t* d_dst_tok_off, int64_t* d_shard_tok_off,
                       int32_t* d_shard_mb_off, int32_t* d_mb_seq_off, int32_t* d_cu_seqlens,
                       int32_t* d_n_mb, const Workspace& ws, int32_t* d_status, hipStream_t st);

hipError_t launch_gather(int32_t n_seq, const FieldTable& ft, int64_t dst_capacity,
                         const int64_t* d_dst_tok_off, const Workspace& ws, hipStream_t st);

}  // namespace dc
