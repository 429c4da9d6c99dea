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
constexpr int32_t REL_FAR = 1 << 30;            // "starts beyond this tile" in tile-relative tokens

struct GatherArgs {
    int32_t        n_seq;
    int32_t        n_tiles;
    int64_t        capacity;
    const int64_t* dst_tok_off;
    const int64_t* slot_src_off;
    const int32_t* slot_len;
    const int32_t* slot_shard;
    const int32_t* tile_first;
};

// A batch of slot descriptors of the tile being moved.  Token positions are relative to
// the tile's first token, so all searching is 32-bit.
struct SegLds {
    int32_t start[NSEG];           // first destination token of the slot (REL_FAR: none / beyond the tile)
    int32_t lensh[NSEG];           // length | rollout shard << 26
    int64_t src[NSEG];             // source element offset inside the rollout shard
};
__device__ __forceinline__ int32_t seg_len(int32_t lensh) { return lensh & ((1 << 26) - 1); }
__device__ __forceinline__ int32_t seg_shard(int32_t lensh) { return lensh >> 26; }

// Largest k in [0, n) with start[k] <= tok, or -1.
__device__ __forceinline__ int find_seg(const int32_t* start, int n, int32_t tok) {
    int lo = 0, hi = n;                       // first k with start[k] > tok
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (start[mid] <= tok) lo = mid + 1; else hi = mid;
    }
    return lo - 1;
}

// Number of entries with start[k] < bound (start is non-decreasing).
__device__ __forceinline__ int count_below(const int32_t* start, int n, int32_t bound) {
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (start[mid] < bound) lo = mid + 1; else hi = mid;
    }
    return lo;
}

template <int ES>
__device__ __forceinline__ uint32_t load_elem(const char* s) {
    if (ES == 4) return *reinterpret_cast<const uint32_t*>(s);
    if (ES == 2) return *reinterpret_cast<const uint16_t*>(s);
    return *reinterpret_cast<const uint8_t*>(s);
}
template <int ES>
__device__ __forceinline__ void store_elem(char* d, uint32_t v) {
    if (ES == 4) *reinterpret_cast<uint32_t*>(d) = v;
    else if (ES == 2) *reinterpret_cast<uint16_t*>(d) = (uint16_t)v;
    else *reinterpret_cast<uint8_t*>(d) = (uint8_t)v;
}

// Where one 16-byte destination chunk comes from.  Shared by all fields of one element size.
struct Chunk {
    int32_t mode;      // 0: not mine in this pass, 1: inside one slot, 2: element by element; | shard << 2
    int64_t elem;      // mode 1: source element index of the chunk's first token
};

template <int TPC>
__device__ __forceinline__ Chunk classify(const SegLds& sg, int n_all, int chunk, int32_t tile_len,
                                          int32_t pass_begin, int32_t pass_end) {
    Chunk c;
    const int32_t c0 = chunk * TPC;
    c.mode = 0; c.elem = 0;
    if (c0 >= pass_begin && c0 < pass_end) {
        const int k = find_seg(sg.start, n_all, c0);
        c.mode = 2;
        if (k >= 0) {
            const int32_t st = sg.start[k], ls = sg.lensh[k];
            if (c0 + TPC <= st + seg_len(ls) && c0 + TPC <= tile_len) {
                c.mode = 1 | (seg_shard(ls) << 2);
                c.elem = sg.src[k] + (c0 - st);
            }
        }
    }
    return c;
}

// 16 source bytes starting at byte address a (a multiple of ES): aligned-down dword loads.
template <int ES>
__device__ __forceinline__ void load_chunk(const char* a, u32x4& v, uint32_t& x) {
    if (ES == 4) {
        v = load16_a4(a);
        x = 0;
    } else {
        const uintptr_t u = reinterpret_cast<uintptr_t>(a);
        const char* a4 = reinterpret_cast<const char*>(u & ~uintptr_t(3));
        v = load16_a4(a4);
        x = (u & 3) ? load4(a4 + 16) : 0u;
    }
}
__device__ __forceinline__ u32x4 realign(u32x4 v, uint32_t x, uint32_t sh) {
    u32x4 o;
    o.x = __builtin_amdgcn_alignbyte(v.y, v.x, sh);
    o.y = __builtin_amdgcn_alignbyte(v.z, v.y, sh);
    o.z = __builtin_amdgcn_alignbyte(v.w, v.z, sh);
    o.w = __builtin_amdgcn_alignbyte(x, v.w, sh);
    return o;
}

// 16-byte chunks of a tile per element size, and how many of them each lane owns
constexpr int N4 = GATHER_TILE / 4, N2 = GATHER_TILE / 8, N1 = GATHER_TILE / 16;
constexpr int U4 = (N4 + GATHER_BLOCK - 1) / GATHER_BLOCK;
constexpr int U2 = (N2 + GATHER_BLOCK - 1) / GATHER_BLOCK;
constexpr int U1 = (N1 + GATHER_BLOCK - 1) / GATHER_BLOCK;

struct FieldLds {
    const char* base[DC_MAX_FIELDS][DC_MAX_SRC_SHARDS];
    char*       dst[DC_MAX_FIELDS];
    int32_t     es[DC_MAX_FIELDS];
    int32_t     cls_nf[3];                       // fields of element size 4, 2, 1
    int32_t     cls_field[3][DC_MAX_FIELDS];
};

// Chunks that cannot take the one-load-one-store path (they cross a slot boundary,
// padding or the arena end), per element-size class.  Their elements are copied one
// per lane afterwards, so a boundary costs one memory round trip, not one per element.
struct BoundaryLds {
    int32_t  count[3];
    uint16_t chunk[3][GATHER_TILE / 4];
};

// Element `tok` (tile-relative) of a boundary chunk: find its slot, copy it.
template <int ES>
__device__ __forceinline__ void move_element(const SegLds& sg, int n_all, int32_t tok, int32_t tile_len,
                                             int64_t tile_begin, char* dst, const char* const* src_base) {
    if (tok >= tile_len) return;
    const int k = find_seg(sg.start, n_all, tok);
    if (k < 0) return;
    const int32_t st = sg.start[k], ls = sg.lensh[k];
    if (tok >= st + seg_len(ls)) return;
    store_elem<ES>(dst + (tile_begin + tok) * ES,
                   load_elem<ES>(src_base[seg_shard(ls)] + (sg.src[k] + (tok - st)) * ES));
}

// Descriptors of slots seg_base + lane and (lanes < SEG_AHEAD) seg_base + SEG_BATCH + lane,
// relative to the tile that starts at token tile_begin.
struct SlotRegs {
    int32_t st[2], ls[2];
    int64_t so[2];
};

__device__ __forceinline__ void load_slots(const GatherArgs& a, int seg_base, int64_t tile_begin, SlotRegs& r) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int64_t j = (int64_t)seg_base + q * SEG_BATCH + (int)threadIdx.x;
        r.st[q] = REL_FAR; r.so[q] = 0; r.ls[q] = 0;
        if ((q == 0 || threadIdx.x < SEG_AHEAD) && seg_base >= 0 && j < a.n_seq) {
            const int64_t d = a.dst_tok_off[j] - tile_begin;
            r.st[q] = (int32_t)max((int64_t)-REL_FAR, min((int64_t)REL_FAR, d));
            r.so[q] = a.slot_src_off[j];
            r.ls[q] = a.slot_len[j] | (a.slot_shard[j] << 26);
        }
    }
}

__device__ __forceinline__ void stage_slots(SegLds& sg, const SlotRegs& r) {
    static_assert(SEG_BATCH == GATHER_BLOCK, "one descriptor per lane plus the look-ahead");
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int k = q * SEG_BATCH + threadIdx.x;
        if (q == 0 || threadIdx.x < SEG_AHEAD) { sg.start[k] = r.st[q]; sg.src[k] = r.so[q]; sg.lensh[k] = r.ls[q]; }
    }
}

// One destination tile, all fields.  On entry the first batch of slot descriptors is
// staged in sg and a barrier has made it (and bl.count = 0) visible.
__device__ __forceinline__ void move_tile(const GatherArgs& a, SegLds& sg, const FieldLds& fl, BoundaryLds& bl,
                                          int nf, int seg_base, int64_t tile_begin, int32_t tile_len) {
    const int tid = threadIdx.x;
    int32_t pass_begin = 0;
    for (;;) {
        const int n_all = count_below(sg.start, NSEG, tile_len);
        const bool more = n_all > SEG_BATCH;               // slot SEG_BATCH also starts inside the tile
        const int32_t pass_end = more ? sg.start[SEG_BATCH] : tile_len;

        // one lookup per element size, shared by every field of that size
        Chunk c4[U4], c2[U2], c1[U1];
#pragma unroll
        for (int u = 0; u < U4; ++u) {
            const int ch = tid + u * GATHER_BLOCK;
            c4[u] = classify<4>(sg, n_all, ch, tile_len, pass_begin, pass_end);
            if (ch >= N4) c4[u].mode = 0;
            if (c4[u].mode == 2) bl.chunk[0][atomicAdd(&bl.count[0], 1)] = (uint16_t)ch;
        }
#pragma unroll
        for (int u = 0; u < U2; ++u) {
            const int ch = tid + u * GATHER_BLOCK;
            c2[u] = classify<8>(sg, n_all, ch, tile_len, pass_begin, pass_end);
            if (ch >= N2) c2[u].mode = 0;
            if (c2[u].mode == 2) bl.chunk[1][atomicAdd(&bl.count[1], 1)] = (uint16_t)ch;
        }
#pragma unroll
        for (int u = 0; u < U1; ++u) {
            const int ch = tid + u * GATHER_BLOCK;
            c1[u] = classify<16>(sg, n_all, ch, tile_len, pass_begin, pass_end);
            if (ch >= N1) c1[u].mode = 0;
            if (c1[u].mode == 2) bl.chunk[2][atomicAdd(&bl.count[2], 1)] = (uint16_t)ch;
        }
        __syncthreads();

        // ---- chunks inside one slot: one field at a time, loads then stores ----
        for (int f = 0; f < nf; ++f) {
            const int es = fl.es[f];
            char* dst = fl.dst[f] + tile_begin * es;
            if (es == 4) {
                u32x4 v[U4];
                uint32_t unused;
#pragma unroll
                for (int u = 0; u < U4; ++u)
                    if (c4[u].mode & 1) load_chunk<4>(fl.base[f][c4[u].mode >> 2] + c4[u].elem * 4, v[u], unused);
#pragma unroll
                for (int u = 0; u < U4; ++u)
                    if (c4[u].mode & 1) store16(dst + (tid + u * GATHER_BLOCK) * 16, v[u]);
            } else if (es == 2) {
                u32x4 v[U2];
                uint32_t x[U2], sh[U2];
#pragma unroll
                for (int u = 0; u < U2; ++u)
                    if (c2[u].mode & 1) {
                        const char* p = fl.base[f][c2[u].mode >> 2] + c2[u].elem * 2;
                        sh[u] = reinterpret_cast<uintptr_t>(p) & 3;
                        load_chunk<2>(p, v[u], x[u]);
                    }
#pragma unroll
                for (int u = 0; u < U2; ++u)
                    if (c2[u].mode & 1) store16(dst + (tid + u * GATHER_BLOCK) * 16, realign(v[u], x[u], sh[u]));
            } else {
                u32x4 v[U1];
                uint32_t x[U1], sh[U1];
#pragma unroll
                for (int u = 0; u < U1; ++u)
                    if (c1[u].mode & 1) {
                        const char* p = fl.base[f][c1[u].mode >> 2] + c1[u].elem;
                        sh[u] = reinterpret_cast<uintptr_t>(p) & 3;
                        load_chunk<1>(p, v[u], x[u]);
                    }
#pragma unroll
                for (int u = 0; u < U1; ++u)
                    if (c1[u].mode & 1) store16(dst + (tid + u * GATHER_BLOCK) * 16, realign(v[u], x[u], sh[u]));
            }
        }
        // ---- boundary chunks: one element per lane and step ----
        {
            const int n4 = bl.count[0] * 4 * fl.cls_nf[0];
            const int n2 = bl.count[1] * 8 * fl.cls_nf[1];
            const int n1 = bl.count[2] * 16 * fl.cls_nf[2];
            for (int wi = tid; wi < n4 + n2 + n1; wi += GATHER_BLOCK) {
                if (wi < n4) {
                    const int e = wi & 3, q = wi >> 2, nfc = fl.cls_nf[0];
                    const int f = fl.cls_field[0][q % nfc];
                    const int32_t tok = (int32_t)bl.chunk[0][q / nfc] * 4 + e;
                    move_element<4>(sg, n_all, tok, tile_len, tile_begin, fl.dst[f], fl.base[f]);
                } else if (wi < n4 + n2) {
                    const int w2 = wi - n4;
                    const int e = w2 & 7, q = w2 >> 3, nfc = fl.cls_nf[1];
                    const int f = fl.cls_field[1][q % nfc];
                    const int32_t tok = (int32_t)bl.chunk[1][q / nfc] * 8 + e;
                    move_element<2>(sg, n_all, tok, tile_len, tile_begin, fl.dst[f], fl.base[f]);
                } else {
                    const int w1 = wi - n4 - n2;
                    const int e = w1 & 15, q = w1 >> 4, nfc = fl.cls_nf[2];
                    const int f = fl.cls_field[2][q % nfc];
                    const int32_t tok = (int32_t)bl.chunk[2][q / nfc] * 16 + e;
                    move_element<1>(sg, n_all, tok, tile_len, tile_begin, fl.dst[f], fl.base[f]);
                }
            }
        }
        if (!more) break;
        // rare: more than SEG_BATCH slots start inside this tile - next batch, loaded in place
        seg_base += SEG_BATCH;
        pass_begin = pass_end;
        __syncthreads();
        SlotRegs r;
        load_slots(a, seg_base, tile_begin, r);
        stage_slots(sg, r);
        if (tid < 3) bl.count[tid] = 0;
        __syncthreads();
    }
}

__global__ __launch_bounds__(GATHER_BLOCK) void gather_kernel(GatherArgs a, FieldTable ft) {
    __shared__ SegLds sg;
    __shared__ FieldLds fl;
    __shared__ BoundaryLds bl;
    const int tid = threadIdx.x;

    const int64_t tile_begin = (int64_t)blockIdx.x * GATHER_TILE;
    const int64_t left = a.capacity - tile_begin;
    const int32_t tile_len = (int32_t)(left < GATHER_TILE ? left : GATHER_TILE);
    if (tile_len <= 0) return;
    const int seg_base = a.tile_first[blockIdx.x];
    if (seg_base < 0 || seg_base >= a.n_seq) return;       // nothing reaches into this tile

    SlotRegs r;
    load_slots(a, seg_base, tile_begin, r);
    if (tid < DC_MAX_FIELDS * DC_MAX_SRC_SHARDS) {
        const int f = tid / DC_MAX_SRC_SHARDS, s = tid % DC_MAX_SRC_SHARDS;
        fl.base[f][s] = (f < ft.n_fields && s < ft.n_src) ? ft.f[f].src[s] : nullptr;
        if (s == 0) { fl.dst[f] = ft.f[f].dst; fl.es[f] = ft.f[f].elem_bytes; }
    }
    if (tid < 3) {
        const int es = 4 >> tid;
        int n = 0;
        for (int f = 0; f < ft.n_fields; ++f)
            if (ft.f[f].elem_bytes == es) fl.cls_field[tid][n++] = f;
        fl.cls_nf[tid] = n;
        bl.count[tid] = 0;
    }
    stage_slots(sg, r);
    __syncthreads();
    move_tile(a, sg, fl, bl, ft.n_fields, seg_base, tile_begin, tile_len);
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
    a.n_tiles = (int32_t)ws.n_tiles;
    hipLaunchKernelGGL(gather_kernel, dim3((unsigned)ws.n_tiles), dim3(GATHER_BLOCK), 0, st, a, ft);
    return hipGetLastError();
}

}  // namespace dc
