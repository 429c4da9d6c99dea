// Segmented gather: rollout layout -> packed training layout (Sec. 6, "Distributed
// Databuffer": re-partitioning of a stage's outputs when the next stage's DP size
// differs).  HBM-bound; every destination byte is written once with aligned
// 16-byte stores, every source byte is read once.
//
// Work decomposition: the destination token axis is cut into tiles of GATHER_TILE
// tokens; one workgroup owns one tile for ALL fields, so no two workgroups ever
// write the same cache line and the slot lookup is shared by the fields.  A tile's
// slots are staged in LDS (start, length, source offset, rollout shard); each lane
// then owns 16-byte destination chunks, finds the slot of its chunk's first token
// by binary search in LDS and
//   - if the chunk lies inside one slot: one (mis)aligned 16-byte source load
//     (plus one dword and a byte funnel shift for 1- and 2-byte fields) and one
//     aligned 16-byte store;
//   - else (slot boundary, padding): element by element.
#include "dc_device.h"
#include "dc_internal.h"

namespace dc {

constexpr int GATHER_BLOCK = 256;
constexpr int NSEG = SEG_BATCH + SEG_AHEAD;

struct GatherArgs {
    int32_t        n_seq;
    int64_t        capacity;
    const int64_t* dst_tok_off;
    const int64_t* slot_src_off;
    const int32_t* slot_len;
    const int32_t* slot_shard;
    const int32_t* tile_first;
};

struct SegLds {
    int64_t start[NSEG];
    int64_t src[NSEG];
    int32_t len[NSEG];
    int32_t shard[NSEG];
};

// Largest k in [0, n) with start[k] <= tok, or -1.
__device__ __forceinline__ int find_seg(const int64_t* start, int n, int64_t tok) {
    int lo = 0, hi = n;                       // first k with start[k] > tok
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (start[mid] <= tok) lo = mid + 1; else hi = mid;
    }
    return lo - 1;
}

// Number of entries with start[k] < bound (start is non-decreasing).
__device__ __forceinline__ int count_below(const int64_t* start, int n, int64_t bound) {
    int lo = 0, hi = n;
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (start[mid] < bound) lo = mid + 1; else hi = mid;
    }
    return lo;
}

template <int ES>
__device__ __forceinline__ void copy_elem(char* d, const char* s) {
    if (ES == 4) *reinterpret_cast<uint32_t*>(d) = *reinterpret_cast<const uint32_t*>(s);
    else if (ES == 2) *reinterpret_cast<uint16_t*>(d) = *reinterpret_cast<const uint16_t*>(s);
    else *reinterpret_cast<uint8_t*>(d) = *reinterpret_cast<const uint8_t*>(s);
}

// All chunks of one field inside the current pass of the tile.
template <int ES>
__device__ __forceinline__ void copy_field(const SegLds& sg, int n_all, char* dst, const char* const* src_base,
                                           int64_t tile_begin, int64_t tile_end,
                                           int64_t pass_begin, int64_t pass_end) {
    constexpr int TPC = 16 / ES;                          // tokens per 16-byte chunk
    constexpr int U = GATHER_TILE / TPC / GATHER_BLOCK;   // chunks per lane: 4, 2, 1
    static_assert(U >= 1, "tile too small");
    u32x4 v[U];
    uint32_t x[U];
    int mode[U];
    int seg[U];
    const char* sp[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c0 = tile_begin + (int64_t)(threadIdx.x + u * GATHER_BLOCK) * TPC;
        mode[u] = 0;
        seg[u] = -1;
        sp[u] = nullptr;
        if (c0 >= pass_begin && c0 < pass_end) {
            const int k = find_seg(sg.start, n_all, c0);
            seg[u] = k;
            mode[u] = 2;
            if (k >= 0) {
                const int64_t st = sg.start[k];
                if (c0 + TPC <= st + sg.len[k] && c0 + TPC <= tile_end) {
                    mode[u] = 1;
                    sp[u] = src_base[sg.shard[k]] + (sg.src[k] + (c0 - st)) * ES;
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (mode[u] == 1) {
            if (ES == 4) {
                v[u] = load16_a4(sp[u]);
            } else {
                const uintptr_t a = reinterpret_cast<uintptr_t>(sp[u]);
                const char* a4 = reinterpret_cast<const char*>(a & ~uintptr_t(3));
                v[u] = load16_a4(a4);
                x[u] = (a & 3) ? load4(a4 + 16) : 0u;
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c0 = tile_begin + (int64_t)(threadIdx.x + u * GATHER_BLOCK) * TPC;
        if (mode[u] == 1) {
            u32x4 o = v[u];
            if (ES != 4) {
                const uint32_t sh = reinterpret_cast<uintptr_t>(sp[u]) & 3;
                o.x = __builtin_amdgcn_alignbyte(v[u].y, v[u].x, sh);
                o.y = __builtin_amdgcn_alignbyte(v[u].z, v[u].y, sh);
                o.z = __builtin_amdgcn_alignbyte(v[u].w, v[u].z, sh);
                o.w = __builtin_amdgcn_alignbyte(x[u], v[u].w, sh);
            }
            store16(dst + c0 * ES, o);
        } else if (mode[u] == 2) {
            int k = seg[u];
            for (int e = 0; e < TPC; ++e) {
                const int64_t tok = c0 + e;
                if (tok >= tile_end) break;
                while (k + 1 < n_all && sg.start[k + 1] <= tok) ++k;
                if (k >= 0) {
                    const int64_t st = sg.start[k];
                    if (tok >= st && tok < st + sg.len[k])
                        copy_elem<ES>(dst + tok * ES, src_base[sg.shard[k]] + (sg.src[k] + (tok - st)) * ES);
                }
            }
        }
    }
}

__global__ __launch_bounds__(GATHER_BLOCK) void gather_kernel(GatherArgs a, FieldTable ft) {
    __shared__ SegLds sg;
    __shared__ const char* s_base[DC_MAX_FIELDS][DC_MAX_SRC_SHARDS];

    const int64_t tile_begin = (int64_t)blockIdx.x * GATHER_TILE;
    const int64_t tile_end = min(tile_begin + (int64_t)GATHER_TILE, a.capacity);
    if (tile_begin >= tile_end) return;
    int seg_base = a.tile_first[blockIdx.x];
    if (seg_base < 0 || seg_base >= a.n_seq) return;       // nothing reaches into this tile

    if (threadIdx.x < DC_MAX_FIELDS * DC_MAX_SRC_SHARDS) {
        const int f = threadIdx.x / DC_MAX_SRC_SHARDS, s = threadIdx.x % DC_MAX_SRC_SHARDS;
        s_base[f][s] = (f < ft.n_fields && s < ft.n_src) ? ft.f[f].src[s] : nullptr;
    }

    int64_t pass_begin = tile_begin;
    for (;;) {
        for (int k = threadIdx.x; k < NSEG; k += GATHER_BLOCK) {
            const int64_t j = (int64_t)seg_base + k;
            int64_t st = INT64_MAX, so = 0;
            int32_t ln = 0, sh = 0;
            if (j < a.n_seq) {
                st = a.dst_tok_off[j];
                so = a.slot_src_off[j];
                ln = a.slot_len[j];
                sh = a.slot_shard[j];
            }
            sg.start[k] = st; sg.src[k] = so; sg.len[k] = ln; sg.shard[k] = sh;
        }
        __syncthreads();
        const int n_all = count_below(sg.start, NSEG, tile_end);
        const bool more = n_all > SEG_BATCH;               // slot SEG_BATCH also starts inside the tile
        const int64_t pass_end = more ? sg.start[SEG_BATCH] : tile_end;

        for (int f = 0; f < ft.n_fields; ++f) {
            char* dst = ft.f[f].dst;
            const int es = ft.f[f].elem_bytes;
            if (es == 4) copy_field<4>(sg, n_all, dst, s_base[f], tile_begin, tile_end, pass_begin, pass_end);
            else if (es == 2) copy_field<2>(sg, n_all, dst, s_base[f], tile_begin, tile_end, pass_begin, pass_end);
            else copy_field<1>(sg, n_all, dst, s_base[f], tile_begin, tile_end, pass_begin, pass_end);
        }
        if (!more) break;
        seg_base += SEG_BATCH;
        pass_begin = pass_end;
        __syncthreads();
    }
}

hipError_t launch_gather(int32_t n_seq, const FieldTable& ft, int64_t dst_capacity,
                         const int64_t* d_dst_tok_off, const Workspace& ws, hipStream_t st) {
    if (n_seq == 0 || ft.n_fields == 0 || ws.n_tiles == 0) return hipSuccess;
    GatherArgs a;
    a.n_seq = n_seq;
    a.capacity = dst_capacity;
    a.dst_tok_off = d_dst_tok_off;
    a.slot_src_off = ws.slot_src_off;
    a.slot_len = ws.slot_len;
    a.slot_shard = ws.slot_shard;
    a.tile_first = ws.tile_first;
    hipLaunchKernelGGL(gather_kernel, dim3((unsigned)ws.n_tiles), dim3(GATHER_BLOCK), 0, st, a, ft);
    return hipGetLastError();
}

}  // namespace dc
