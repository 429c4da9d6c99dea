// Reverse path: packed training layout -> rollout layout, for per-token fields a stage
// running in the training layout produced (the collect / concat side of a stage transition,
// App. B Table 2; Sec. 6 "Distributed Databuffer" moves data between stages in both
// directions).
//
// A scatter by destination would write the rollout buffers in sequence-random order, which
// costs twice what random reads cost.  Instead the rollout layout is treated as the
// DESTINATION of a gather: sequence i of rollout shard s is "slot" i of that shard, it starts
// at its rollout offset and comes from element dst_tok_off[slot of i] of the training arena.
// Two small kernels write those per-sequence descriptors, one launch builds the granule tables
// of every rollout buffer's token axis, and one launch of the gather's tile mover (the rollout
// buffers being destination segments of one grid) moves the data: linear, aligned 16-byte
// stores into the rollout buffers, one (mis)aligned load per chunk from the arena.
#include "dc_device.h"
#include "dc_internal.h"

namespace dc {

constexpr int SCAT_BLOCK = 256;

struct ScatArgs {
    int32_t        n_seq;
    int64_t        capacity;         // elements of every training arena
    const int64_t* src_tok_off;      // rollout offset of every sequence
    const int32_t* seq_len;
    const int32_t* perm;
    const int64_t* dst_tok_off;      // arena offset of every slot
    int64_t*       r_dst_off;
    int64_t*       r_src_off;
    int32_t*       r_len;
    int32_t*       r_shard;
    int32_t*       status;
};

__device__ __forceinline__ int rollout_shard(const SourceDesc& sd, int i) {
    int sh = 0;                                          // seq_off[s] = N from s = n_src on
    if (sd.n_src > 1) {
#pragma unroll
        for (int s = 1; s < DC_MAX_SRC_SHARDS; ++s) sh += i >= sd.seq_off[s] ? 1 : 0;
    }
    return sh;
}
__device__ __forceinline__ int64_t shard_tokens(const SourceDesc& sd, int sh) {
    int64_t t = sd.tokens[0];
#pragma unroll
    for (int s = 1; s < DC_MAX_SRC_SHARDS; ++s) t = sh == s ? sd.tokens[s] : t;
    return t;
}

// One lane per sequence: its start in the rollout buffer (clamped into the buffer), nothing to
// move yet; one lane per rollout shard: the end of the buffer behind its last sequence.
__global__ __launch_bounds__(SCAT_BLOCK) void scatter_init_kernel(ScatArgs a, SourceDesc sd) {
    const int i = blockIdx.x * SCAT_BLOCK + threadIdx.x;
    if (i < sd.n_src) a.r_dst_off[sd.seq_off[i + 1] + i] = sd.tokens[i];
    if (i >= a.n_seq) return;
    const int sh = rollout_shard(sd, i);
    const int64_t so = a.src_tok_off[i];
    a.r_dst_off[i + sh] = max((int64_t)0, min(so, shard_tokens(sd, sh)));
    a.r_src_off[i] = 0;
    a.r_len[i] = 0;
    a.r_shard[i] = 0;
}

// One lane per slot j: the sequence it holds gets its length and its place in the arena, if every
// check passes (the rollout side is written, so nothing unchecked may steer a store).
__global__ __launch_bounds__(SCAT_BLOCK) void scatter_slots_kernel(ScatArgs a, SourceDesc sd) {
    const int j = blockIdx.x * SCAT_BLOCK + threadIdx.x;
    const int N = a.n_seq;
    if (j >= N) return;
    const int32_t i = a.perm[j];
    if (i < 0 || i >= N) { set_status(a.status, DC_ERR_BAD_LAYOUT); return; }
    const int sh = rollout_shard(sd, i);
    const int32_t ln = a.seq_len[i];
    const int64_t so = a.src_tok_off[i];
    const int64_t from = a.dst_tok_off[j];
    if (ln <= 0 || ln > DC_MAX_SEQ_LEN) { set_status(a.status, DC_ERR_ZERO_LENGTH_SEQ); return; }
    const bool last_in_shard = i + 1 >= sd.seq_off[sh + 1];
    const int64_t next = last_in_shard ? shard_tokens(sd, sh) : a.src_tok_off[i + 1];
    if (so < 0 || so + ln > shard_tokens(sd, sh) || so + ln > next) { set_status(a.status, DC_ERR_BAD_LAYOUT); return; }
    if (from < 0 || from + ln > a.capacity) { set_status(a.status, DC_ERR_OVERFLOW); return; }
    // the first slot that claims a sequence places it; a second one means perm is not a permutation (and, N
    // entries being in range, that some sequence is placed by none).  One of the claimants' offsets is used:
    // outputs are unspecified once the status is set, but every access stays inside the buffers.
    if (atomicCAS(a.r_len + i, 0, ln) != 0) { set_status(a.status, DC_ERR_BAD_LAYOUT); return; }
    a.r_src_off[i] = from;
}

BackSegs make_back_segs(const SourceDesc& src) {
    BackSegs b;
    b.n_seg = src.n_src;
    uint32_t tiles = 0;
    int64_t gran = 0;
    for (int s = 0; s < DC_MAX_SRC_SHARDS; ++s) {
        const bool live = s < src.n_src && src.seq_off[s + 1] > src.seq_off[s] && src.tokens[s] > 0;
        b.first_seq[s] = s < src.n_src ? src.seq_off[s] : 0;
        b.n_seq[s] = live ? src.seq_off[s + 1] - src.seq_off[s] : 0;
        b.tokens[s] = live ? src.tokens[s] : 0;
        b.gran_base[s] = gran;
        if (live) {
            tiles += (uint32_t)((src.tokens[s] + GATHER_TILE_TOKENS - 1) / GATHER_TILE_TOKENS);
            // whole tiles plus the padding the tile mover's table loads need; a multiple of 4 entries
            gran += ((src.tokens[s] + GATHER_GRAN - 1) / GATHER_GRAN + GRAN_TABLE_PAD + 3) / 4 * 4;
        }
        b.tile_end[s] = tiles;
    }
    b.gran_base[DC_MAX_SRC_SHARDS] = gran;
    return b;
}

ScatterWorkspace carve_scatter_workspace(void* base, int32_t n_seq, const SourceDesc& src) {
    auto round_up = [](size_t x, size_t a) { return (x + a - 1) / a * a; };
    ScatterWorkspace w;
    const size_t n = (size_t)(n_seq > 0 ? n_seq : 0);
    char* p = static_cast<char*>(base);
    size_t off = 0;
    w.r_dst_off = reinterpret_cast<int64_t*>(p + off); off += round_up((n + DC_MAX_SRC_SHARDS) * sizeof(int64_t), 256);
    w.r_src_off = reinterpret_cast<int64_t*>(p + off); off += round_up(n * sizeof(int64_t), 256);
    w.r_len = reinterpret_cast<int32_t*>(p + off);     off += round_up(n * sizeof(int32_t), 256);
    w.r_shard = reinterpret_cast<int32_t*>(p + off);   off += round_up(n * sizeof(int32_t), 256);
    w.n_gran_all = make_back_segs(src).gran_base[DC_MAX_SRC_SHARDS];
    w.gran_first = reinterpret_cast<int32_t*>(p + off); off += round_up((size_t)w.n_gran_all * sizeof(int32_t), 256);
    w.gran_rec = reinterpret_cast<GranRec*>(p + off);   off += round_up((size_t)w.n_gran_all * sizeof(GranRec), 256);
    w.bytes = off + 256;
    return w;
}

hipError_t launch_scatter(int32_t n_seq, const SourceDesc& src, const int64_t* d_src_tok_off,
                          const int32_t* d_seq_len, const int32_t* d_perm, const FieldTable& ft,
                          int64_t dst_capacity, const int64_t* d_dst_tok_off, const ScatterWorkspace& ws,
                          int32_t* d_status, hipStream_t st) {
    if (n_seq == 0 || ft.n_fields == 0) return hipSuccess;
    ScatArgs a;
    a.n_seq = n_seq; a.capacity = dst_capacity; a.src_tok_off = d_src_tok_off; a.seq_len = d_seq_len;
    a.perm = d_perm; a.dst_tok_off = d_dst_tok_off; a.r_dst_off = ws.r_dst_off; a.r_src_off = ws.r_src_off;
    a.r_len = ws.r_len; a.r_shard = ws.r_shard; a.status = d_status;
    const unsigned grid = (unsigned)((n_seq + SCAT_BLOCK - 1) / SCAT_BLOCK);
    hipLaunchKernelGGL(scatter_init_kernel, dim3(grid), dim3(SCAT_BLOCK), 0, st, a, src);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(scatter_slots_kernel, dim3(grid), dim3(SCAT_BLOCK), 0, st, a, src);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const BackSegs bs = make_back_segs(src);
    e = launch_records_back(bs, ws, st);
    if (e != hipSuccess) return e;
    return launch_gather_back(bs, ft, ws, st);
}

}  // namespace dc
