// Host-side declarations shared by the API layer and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include "../../include/dc.h"

namespace dc {

// Token granularity of the per-granule tables the plan leaves in the workspace.  A
// 16-byte chunk of any field (4, 8 or 16 tokens) never crosses a granule boundary.
constexpr int GATHER_GRAN = 1024;
// The per-granule tables are longer than the arena needs, so a gather workgroup can read
// the entries of a whole tile (and a few more) without a bounds test.
constexpr int GRAN_TABLE_PAD = 16;
constexpr int GRAN_PER_TILE = 4;                 // granules (waves) per gather tile
constexpr int GATHER_TILE_TOKENS = GRAN_PER_TILE * GATHER_GRAN;
// Slot descriptors kept inline per granule; granules that more slots reach into are
// served from the per-slot arrays instead.
constexpr int REC_SLOTS = 4;
constexpr int32_t REL_FAR = 1 << 30;            // "no slot" / "beyond this granule" in relative tokens
constexpr int LENSH_SHIFT = 26;                 // length | rollout shard << 26
static_assert(DC_MAX_SEQ_LEN < (1 << LENSH_SHIFT) && DC_MAX_SRC_SHARDS <= (1 << (31 - LENSH_SHIFT)),
              "a length and a rollout shard share one non-negative 32-bit word");

// The first REC_SLOTS slots that reach into a granule, relative to the granule's first
// token.  Unused entries have start = REL_FAR.  64 bytes: one 16-dword scalar load.
struct GranEntry {
    int32_t start;           // first destination token of the slot minus the granule's first token (may be < 0)
    int32_t lensh;           // length | rollout shard << LENSH_SHIFT
    int64_t src_off;         // element offset of the slot's sequence in its rollout shard
};
struct GranRec { GranEntry e[REC_SLOTS]; };

// Tokens of rollout space one advantage workgroup owns.
constexpr int ADV_TILE = 8192;
// Segment descriptors staged in LDS per pass over a tile, plus look-ahead so a
// 16-token chunk that starts in the last owned segment can be finished.
constexpr int SEG_BATCH = 256;
constexpr int SEG_AHEAD = 16;


// Workspace carved by dc_plan for dc_gather: per-slot source descriptors
// (validated, clamped) and, for every granule boundary g * GATHER_GRAN of the
// destination token axis, the first slot that ends after it.
struct Workspace {
    int64_t* slot_src_off;   // [N]   element offset of the slot's sequence in its rollout shard
    int32_t* slot_len;       // [N]   tokens to copy (0 if the slot failed validation)
    int32_t* slot_shard;     // [N]   rollout shard of the slot's sequence
    int32_t* gran_first;     // [n_gran] first slot j with end(j) > g * GATHER_GRAN (N if none); non-decreasing
    GranRec* gran_rec;       // [n_gran]
    int32_t* plan_ok;        // [1] 0 if the plan kernel found the shard table unusable and planned nothing
    int32_t* own_shard_off;  // [DC_MAX_SRC_SHARDS + 1] the rollout shards' sequence offsets, for a plan that keeps them
    int64_t* gpre;           // [N + 1]  } only above DC_MAX_SEQ slots (else null): what plan_kernel keeps in LDS
    int32_t* word_starts;    // [N / 32 + 2]
    int32_t* word_last;      // [N / 32 + 2]
    int64_t  n_gran;         // ceil(capacity / GATHER_GRAN) + GRAN_TABLE_PAD; entries past the arena hold N / no slot
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
    FieldDesc f[DC_MAX_FIELDS + 1];       // one more: the gather that makes the advantage field describes it here
};

hipError_t launch_balance(int32_t n_seq, int32_t n_shards, int32_t cap_eff, const int32_t* d_seq_len,
                          int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                          int64_t* d_shard_load, int32_t* d_status, hipStream_t st);

// The same for DC_MAX_SEQ < n_seq <= DC_MAX_SEQ_LARGE, cap_eff < 2^16; d_ws: 3 * roundup(n_seq, 64) int32 words and
// then sort_large_table_bytes(n_seq) bytes, 256-byte aligned.
hipError_t launch_balance_large(int32_t n_seq, int32_t n_shards, int32_t cap_eff, const int32_t* d_seq_len,
                                int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                                int64_t* d_shard_load, void* d_ws, int32_t* d_status, hipStream_t st);

// Indices by descending length (stable), by many workgroups (sort_large.hip).
size_t sort_large_table_bytes(int32_t n_seq);
hipError_t launch_sort_large(int32_t n_seq, const int32_t* d_seq_len, int32_t* d_idx_a, int32_t* d_idx_b,
                             int32_t* d_sorted_len, uint32_t* d_counts, int32_t* d_status, hipStream_t st);

struct AdvArgs;
hipError_t launch_balance_advantage(int32_t n_seq, int32_t n_shards, int32_t cap_eff, const int32_t* d_seq_len,
                                    int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                                    int64_t* d_shard_load, const AdvArgs& adv, const SourceDesc& src,
                                    int32_t n_groups, int32_t* d_status, hipStream_t st);
hipError_t launch_advantage(int32_t n_seq, const SourceDesc& src, const int64_t* d_src_tok_off,
                            const int32_t* d_seq_len, const float* d_reward, const int32_t* d_group_off,
                            int32_t n_groups, double eps, int32_t ddof,
                            const uint8_t* const* mask_base, float* d_adv_seq, float* const* adv_tok_base,
                            int32_t* d_status, hipStream_t st);

// Arguments of the plan kernels.
struct PlanArgs {
    int32_t n_seq, n_shards, align;
    int64_t budget, capacity;
    const int64_t* src_tok_off;
    const int32_t* seq_len;
    const int32_t* perm;
    const int32_t* shard_seq_off;
    int32_t* own_shard_off;         // not null: the caller gave no shard table; slots_kernel writes the rollout shards'
                                    // one here and shard_seq_off points at it
    int64_t* dst_tok_off;
    int64_t* shard_tok_off;
    int32_t* shard_mb_off;
    int32_t* mb_seq_off;
    int32_t* cu_seqlens;
    int32_t* n_mb;
    int64_t* slot_src_off;
    int32_t* slot_len;
    int32_t* slot_shard;
    int32_t* plan_ok;
    int32_t* status;
    // more than DC_MAX_SEQ slots only (workspace): dense prefix of the slot lengths, and per word of 32 slots
    // the micro-batch starts before it / the last start before it
    int64_t* gpre;
    int32_t* word_starts;
    int32_t* word_last;
};

PlanArgs make_plan_args(const dc_params& prm, const int64_t* d_src_tok_off, const int32_t* d_seq_len,
                        const int32_t* d_perm, const int32_t* d_shard_seq_off, int64_t dst_capacity,
                        int64_t* d_dst_tok_off, int64_t* d_shard_tok_off, int32_t* d_shard_mb_off,
                        int32_t* d_mb_seq_off, int32_t* d_cu_seqlens, int32_t* d_n_mb, const Workspace& ws,
                        int32_t* d_status);

// Granule tables and per-slot source descriptors behind a plan that ran as the balance workgroup's tail
// (p.slot_len holds the slots' lengths, nothing else of the per-slot arrays is filled yet).
hipError_t launch_records_slots(const PlanArgs& p, const SourceDesc& src, const Workspace& ws, hipStream_t st);

// Balance, group advantage and the plan in one launch (workgroup 0: Algorithm 1, then the plan as its tail;
// the other workgroups: the advantage stage).  Needs n_shards in {16, 32, 64}, cap_eff * n_shards == n_seq.
hipError_t launch_balance_plan_advantage(int32_t n_seq, int32_t n_shards, int32_t cap_eff, const int32_t* d_seq_len,
                                         int32_t* d_perm, int32_t* d_shard_seq_off, int32_t* d_shard_of_seq,
                                         int64_t* d_shard_load, const PlanArgs& plan, const AdvArgs& adv,
                                         const SourceDesc& src, int32_t n_groups, int32_t* d_status, hipStream_t st);

// plan_kernel's work for DC_MAX_SEQ < n_seq <= DC_MAX_SEQ_LARGE: one workgroup, the prefix and the per-word
// tables in the workspace instead of the LDS.
hipError_t launch_plan_large(const PlanArgs& a, hipStream_t st);

hipError_t launch_plan(const dc_params& prm, const SourceDesc& src, const int64_t* d_src_tok_off,
                       const int32_t* d_seq_len, const int32_t* d_perm, const int32_t* d_shard_seq_off,
                       int64_t dst_capacity, int64_t* d_dst_tok_off, int64_t* d_shard_tok_off,
                       int32_t* d_shard_mb_off, int32_t* d_mb_seq_off, int32_t* d_cu_seqlens,
                       int32_t* d_n_mb, const Workspace& ws, int32_t* d_status, hipStream_t st);

// begins / ends (each may be null): events that the kernel's dispatch itself updates with the times at which the
// kernel starts and ends on the device.
hipError_t launch_gather(int32_t n_seq, const FieldTable& ft, int64_t dst_capacity,
                         const int64_t* d_dst_tok_off, const Workspace& ws, hipStream_t st,
                         hipEvent_t begins = nullptr, hipEvent_t ends = nullptr);

// launch_gather plus the float32 advantage arena d_adv_tok_dst, made from field mask_field (1-byte
// elements) and the per-sequence advantages; the workgroups that make it also move the mask.
hipError_t launch_gather_advantage(int32_t n_seq, const FieldTable& ft, int mask_field, const int32_t* d_perm,
                                   const float* d_adv_seq, float* d_adv_tok_dst, int64_t dst_capacity,
                                   const int64_t* d_dst_tok_off, const Workspace& ws, hipStream_t st);

// Granule tables (ws.gran_first, ws.gran_rec) from slot starts d_dst_tok_off[0..n_seq] and the
// per-slot descriptors in ws; *ws.plan_ok == 0 makes them empty.
hipError_t launch_records(int32_t n_seq, const int64_t* d_dst_tok_off, const Workspace& ws, hipStream_t st);

// Workspace of the reverse path: the rollout layout seen as a destination.  Sequence i of
// rollout shard s is "slot" i of that shard; r_dst_off has one more entry per shard (its end).
// The granule tables of the rollout buffers lie one behind the other, each padded like the
// forward path's.
struct ScatterWorkspace {
    int64_t* r_dst_off;      // [N + n_src] slot start in the rollout buffer, shard s at index seq_off[s] + s
    int64_t* r_src_off;      // [N] element offset of the sequence in the training arena
    int32_t* r_len;          // [N] tokens to move (0 if a check failed or perm does not place the sequence)
    int32_t* r_shard;        // [N] zeros: the arena is the only "source shard"
    int32_t* gran_first;     // [n_gran_all]
    GranRec* gran_rec;       // [n_gran_all]
    int64_t  n_gran_all;
    size_t   bytes;
};
ScatterWorkspace carve_scatter_workspace(void* base, int32_t n_seq, const SourceDesc& src);

// The rollout buffers as destination segments of one launch: segment s owns tiles
// [tile_end[s-1], tile_end[s]) of the grid and granules [gran_base[s], gran_base[s+1]) of the tables.
struct BackSegs {
    int32_t  n_seg;
    int32_t  first_seq[DC_MAX_SRC_SHARDS];
    int32_t  n_seq[DC_MAX_SRC_SHARDS];
    uint32_t tile_end[DC_MAX_SRC_SHARDS];      // running total; entries from n_seg on repeat the grand total
    int64_t  gran_base[DC_MAX_SRC_SHARDS + 1];
    int64_t  tokens[DC_MAX_SRC_SHARDS];
};
BackSegs make_back_segs(const SourceDesc& src);

hipError_t launch_records_back(const BackSegs& bs, const ScatterWorkspace& ws, hipStream_t st);
hipError_t launch_gather_back(const BackSegs& bs, const FieldTable& ft, const ScatterWorkspace& ws, hipStream_t st);

hipError_t launch_scatter(int32_t n_seq, const SourceDesc& src, const int64_t* d_src_tok_off,
                          const int32_t* d_seq_len, const int32_t* d_perm, const FieldTable& ft,
                          int64_t dst_capacity, const int64_t* d_dst_tok_off, const ScatterWorkspace& ws,
                          int32_t* d_status, hipStream_t st);

hipError_t launch_gae(int32_t n_seq, const SourceDesc& src, const int64_t* d_src_tok_off, const int32_t* d_seq_len,
                      const float* d_reward, const float* const* value_base, const uint8_t* const* mask_base,
                      const float* const* logp_base, const float* const* ref_base, double gamma, double lambda,
                      double kl_coef, float* const* adv_base, float* const* ret_base, int32_t* d_status,
                      hipStream_t st);

}  // namespace dc
