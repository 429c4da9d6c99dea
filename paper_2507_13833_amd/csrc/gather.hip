// Segmented gather: rollout layout -> packed training layout (Sec. 6, "Distributed
// Databuffer": re-partitioning of a stage's outputs when the next stage's DP size
// differs).  HBM-bound; every destination byte is written once with aligned
// 16-byte stores, every source byte is read once.
//
// Work decomposition: FIELD-MAJOR.  The destination token axis is cut into tiles of 4096
// tokens; the grid walks all tiles of field 0, then all tiles of field 1, ...  At any
// moment the chip therefore streams one destination array (and the matching sequences of
// one source array) instead of all fields at once, which keeps DRAM pages open longer than
// a tile that touches every field.  One workgroup owns one tile of one field, one wavefront
// a 1024-token granule of it (1, 2 or 4 16-byte chunks per lane for 1-, 2-, 4-byte
// elements); no two workgroups ever write the same cache line.
//
// Where a chunk comes from:
//   sparse tiles (at most REC_SLOTS slots reach into each granule: the usual case) - every
//     wave works alone: it reads its granule's record (the plan left the first slots of
//     every granule inline) with ONE scalar load, which does not queue behind the bulk
//     traffic in the vector memory pipeline; when one slot covers all 64 chunks of a wave
//     instruction the source address is scalar arithmetic, else every lane selects its
//     slot with a few compares against scalar registers.  No LDS, no barrier;
//   dense tiles (many short sequences) - the tile's slots are staged in LDS and each
//     lane finds its chunk's slot by binary search.
// A chunk inside one slot takes one (mis)aligned 16-byte source load (plus one dword
// and a byte funnel shift for 1- and 2-byte fields) and one aligned 16-byte store;
// a chunk that touches a slot boundary, padding or the arena end is copied element
// by element.
#include <hip/hip_ext.h>
#include "dc_device.h"
#include "dc_internal.h"

namespace dc {

constexpr int GATHER_BLOCK = 256;
constexpr int NSEG = SEG_BATCH + SEG_AHEAD;
static_assert(GRAN_PER_TILE == GATHER_BLOCK / WAVE, "one granule per wave");
constexpr int64_t GATHER_RIDE_MIN_WGS = 8192;                         // ~4 workgroups per wave slot of the chip
constexpr int32_t LEN_MASK = (1 << LENSH_SHIFT) - 1;
static_assert(GATHER_GRAN == WAVE * 16, "a wave covers its granule with 1, 2 or 4 chunks per lane");
static_assert(GRAN_PER_TILE + 1 <= 8, "the tile's slice of the granule table is one 8-dword scalar load");
static_assert(GRAN_TABLE_PAD >= 8, "that load never leaves the table");
static_assert(sizeof(GranEntry) == 16, "one 16-byte load per record entry");
static_assert(SEG_BATCH == GATHER_BLOCK, "one descriptor per lane plus the look-ahead");

struct GatherArgs {
    int32_t        n_seq;
    int64_t        capacity;                     // elements of every destination arena
    const int64_t* dst_tok_off;
    const int64_t* slot_src_off;
    const int32_t* slot_len;
    const int32_t* slot_shard;
    const int32_t* gran_first;                   // padded: whole tiles plus GRAN_PER_TILE + 1 entries
    const GranRec* gran_rec;                     // same length
    uint32_t       tiles;                        // tiles per field
    uint32_t       n_carriers, n_riders;         // fields the grid walks (first in the field table), fields riding along
};

// Slot descriptors of the tile being moved, relative to the tile's first token.
struct SegLds {
    int32_t start[NSEG];           // first destination token of the slot (REL_FAR: none)
    int32_t end[NSEG];             // one past its last token
    int64_t addr[NSEG];            // source byte address of tile-relative token 0 (may lie before the buffer)
};

// Largest k in [0, n) with start[k] <= tok, or -1.
__device__ __forceinline__ int find_seg(const int32_t* start, int n, int32_t tok) {
    int lo = 0, hi = n;                       // first k with start[k] > tok
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (start[mid] <= tok) lo = mid + 1; else hi = mid;
    }
    return lo - 1;
}

// Payload pointers are rebuilt from integers (base + offset arithmetic in scalar registers
// or LDS); typing them as global-address-space pointers keeps the accesses global_load /
// global_store instead of flat ones.
#define DC_GLOBAL __attribute__((address_space(1)))
typedef const DC_GLOBAL char* gptr;
typedef DC_GLOBAL char* gptr_w;

// One element of 1 << lg bytes (lg is uniform).
__device__ __forceinline__ uint32_t load_elem(int lg, gptr s) {
    if (lg == 2) return *reinterpret_cast<const DC_GLOBAL uint32_t*>(s);
    if (lg == 1) return *reinterpret_cast<const DC_GLOBAL uint16_t*>(s);
    return *reinterpret_cast<const DC_GLOBAL uint8_t*>(s);
}
__device__ __forceinline__ void store_elem(int lg, gptr_w d, uint32_t v) {
    if (lg == 2) *reinterpret_cast<DC_GLOBAL uint32_t*>(d) = v;
    else if (lg == 1) *reinterpret_cast<DC_GLOBAL uint16_t*>(d) = (uint16_t)v;
    else *reinterpret_cast<DC_GLOBAL uint8_t*>(d) = (uint8_t)v;
}

typedef DC_GLOBAL u32x4 g_u32x4;
typedef DC_GLOBAL u32x4_a4 g_u32x4_a4;
__device__ __forceinline__ u32x4 gload16_a4(gptr p) {
    return __builtin_nontemporal_load(reinterpret_cast<const g_u32x4_a4*>(p));
}
__device__ __forceinline__ uint32_t gload4(gptr p) {
    return __builtin_nontemporal_load(reinterpret_cast<const DC_GLOBAL uint32_t*>(p));
}
__device__ __forceinline__ void gstore16(gptr_w p, u32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<g_u32x4*>(p));
}
__device__ __forceinline__ void gstore4(gptr_w p, uint32_t v) {
    __builtin_nontemporal_store(v, reinterpret_cast<DC_GLOBAL uint32_t*>(p));
}

// 16 source bytes starting at byte address a (any alignment): dword loads from the address
// rounded down to 4, plus the following dword when a is not a multiple of 4; realign()
// shifts them into place (a no-op for aligned sources, e.g. every 4-byte field).
__device__ __forceinline__ void load_chunk(gptr a, u32x4& v, uint32_t& x) {
    const uintptr_t u = reinterpret_cast<uintptr_t>(a);
    gptr a4 = reinterpret_cast<gptr>(u & ~uintptr_t(3));
    v = gload16_a4(a4);
    x = (u & 3) ? gload4(a4 + 16) : 0u;
}
__device__ __forceinline__ u32x4 realign(u32x4 v, uint32_t x, uint32_t sh) {
    u32x4 o;
    o.x = __builtin_amdgcn_alignbyte(v.y, v.x, sh);
    o.y = __builtin_amdgcn_alignbyte(v.z, v.y, sh);
    o.z = __builtin_amdgcn_alignbyte(v.w, v.z, sh);
    o.w = __builtin_amdgcn_alignbyte(x, v.w, sh);
    return o;
}

// Stage descriptors of slots seg_base + lane and (lanes < SEG_AHEAD) seg_base + SEG_BATCH + lane,
// up to slot seg_last, for the field whose rollout buffers are src[] and the tile that
// starts at token tile_begin.
__device__ __forceinline__ void stage_slots(const GatherArgs& a, SegLds& sg, const char* const* src, int lg,
                                            int seg_base, int seg_last, int64_t tile_begin) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int k = q * SEG_BATCH + (int)threadIdx.x;
        const int j = seg_base + k;
        if (q == 0 || threadIdx.x < SEG_AHEAD) {
            int32_t st = REL_FAR, en = REL_FAR;
            int64_t ad = 0;
            if (j <= seg_last) {
                const int64_t d = a.dst_tok_off[j] - tile_begin;
                st = (int32_t)max((int64_t)-REL_FAR, min((int64_t)REL_FAR, d));
                en = st + a.slot_len[j];
                ad = reinterpret_cast<int64_t>(src[a.slot_shard[j]]) + ((a.slot_src_off[j] - d) << lg);
            }
            sg.start[k] = st; sg.end[k] = en; sg.addr[k] = ad;
        }
    }
}

// One destination tile of one field with element size 1 << lg, slots staged in LDS (whole
// workgroup, barriers inside).  On return every lane has passed a barrier after its last LDS read.
__device__ __forceinline__ void move_tile_dense(const GatherArgs& a, SegLds& sg, const char* const* src, int lg,
                                                char* dst_field, int seg_first, int seg_last, int64_t tile_begin,
                                                int32_t tile_len) {
    const int tpc = 16 >> lg;                              // tokens per 16-byte chunk
    const int tid = threadIdx.x;
    gptr_w dst = reinterpret_cast<gptr_w>(reinterpret_cast<uintptr_t>(dst_field) + (tile_begin << lg));
    int seg_base = seg_first;
    int32_t pass_begin = 0;
    for (;;) {
        stage_slots(a, sg, src, lg, seg_base, seg_last, tile_begin);
        __syncthreads();
        const int n_left = seg_last - seg_base + 1;
        const int n_all = min(n_left, NSEG);
        // more than SEG_BATCH slots left and the next batch's first slot starts inside the tile
        const bool more = n_left > SEG_BATCH && sg.start[SEG_BATCH] < tile_len;
        const int32_t pass_end = more ? sg.start[SEG_BATCH] : tile_len;

#pragma unroll 1
        for (int u = 0; u < (1 << lg); ++u) {              // 1 << lg chunks per lane, one at a time: this path
            const int32_t c0 = (tid + u * GATHER_BLOCK) * tpc;   // is the rare one and must not cost registers
            if (c0 < pass_begin || c0 >= pass_end) continue;
            int k = find_seg(sg.start, n_all, c0);
            if (k >= 0 && c0 + tpc <= sg.end[k] && c0 + tpc <= tile_len) {
                // inside one slot: one load, one store
                gptr ad = reinterpret_cast<gptr>(sg.addr[k] + ((int64_t)c0 << lg));
                u32x4 v;
                uint32_t x;
                load_chunk(ad, v, x);
                gstore16(dst + (tid + u * GATHER_BLOCK) * 16, realign(v, x, (uint32_t)reinterpret_cast<uintptr_t>(ad) & 3u));
            } else {
                // touches a slot boundary, padding or the arena end: per element
                for (int e = 0; e < tpc; ++e) {
                    const int32_t tok = c0 + e;
                    if (tok >= tile_len) break;
                    while (k + 1 < n_all && sg.start[k + 1] <= tok) ++k;
                    if (k >= 0 && tok < sg.end[k])
                        store_elem(lg, dst + ((int64_t)tok << lg),
                                   load_elem(lg, reinterpret_cast<gptr>(sg.addr[k] + ((int64_t)tok << lg))));
                }
            }
        }
        __syncthreads();
        if (!more) break;
        // rare: more than SEG_BATCH slots start inside this tile - next batch
        seg_base += SEG_BATCH;
        pass_begin = pass_end;
    }
}

// ---------------------------------------------------------------- sparse tiles: one wave, no LDS
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
#define DC_CONSTANT __attribute__((address_space(4)))

// Uniform loads through the scalar data cache: they do not queue behind the bulk traffic in
// the vector memory pipeline, and their results land in scalar registers.
__device__ __forceinline__ u32x8 sload8(const void* p) {
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wold-style-cast"
    return *(const DC_CONSTANT u32x8*)p;
#pragma clang diagnostic pop
}
__device__ __forceinline__ u32x16 sload16(const void* p) {
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wold-style-cast"
    return *(const DC_CONSTANT u32x16*)p;
#pragma clang diagnostic pop
}

// One record entry as the selection needs it (all scalar): the slot's first token and end
// relative to the granule, and the source byte address the granule's token 0 would have
// inside the slot.
struct SlotS {
    int32_t st, en;
    int64_t ad;
};

// The elements of one 16-byte chunk that does not lie inside one slot, on their way.
struct BoundaryChunk {
    uint32_t val[16];
    uint32_t ok;             // bit r: element r exists (belongs to a slot, inside the arena) and was loaded
    int32_t  c0;             // the chunk's first token inside the granule
};

template <int LG>
__device__ __forceinline__ void boundary_load(const SlotS (&e)[REC_SLOTS], bool mine, int32_t limit, BoundaryChunk& bc) {
#pragma unroll
    for (int r = 0; r < (16 >> LG); ++r) {
        const int32_t t = bc.c0 + r;
        int32_t e_sel = INT32_MIN;
        int64_t a_sel = 0;
#pragma unroll
        for (int k = 0; k < REC_SLOTS; ++k)
            if (t >= e[k].st) { e_sel = e[k].en; a_sel = e[k].ad; }
        bc.val[r] = 0;
        if (mine && t < e_sel && t < limit) {
            bc.ok |= 1u << r;
            bc.val[r] = load_elem(LG, reinterpret_cast<gptr>(a_sel + ((int64_t)t << LG)));
        }
    }
}

template <int LG>
__device__ __forceinline__ void boundary_store(gptr_w dst, const BoundaryChunk& bc) {
#pragma unroll
    for (int r = 0; r < (16 >> LG); ++r)
        if (bc.ok & (1u << r)) store_elem(LG, dst + ((int64_t)(bc.c0 + r) << LG), bc.val[r]);
}

// The wave's granule (1024 tokens: es chunks per lane) of one tile, served from the granule's
// record.  `limit` = tokens of the granule that exist in the arena (> 0).
// BACK: destination and only source are given (back_dst, back_src) instead of fd's.
template <bool BACK>
__device__ __forceinline__ void move_wave_sparse(const FieldDesc& fd, int n_src, char* back_dst, const char* back_src,
                                                 int lg, const u32x16& rec, int64_t wave_begin, int32_t limit) {
    const int es = 1 << lg;
    const int tpc = 16 >> lg;                              // tokens per 16-byte chunk
    const int tpi = WAVE * tpc;                            // tokens one wave instruction covers
    const int lane = threadIdx.x & (WAVE - 1);
    gptr_w dst = reinterpret_cast<gptr_w>(reinterpret_cast<uintptr_t>(BACK ? back_dst : fd.dst) + (wave_begin << lg));

    SlotS e[REC_SLOTS];
#pragma unroll
    for (int k = 0; k < REC_SLOTS; ++k) {
        const int32_t st = (int32_t)rec[4 * k], ls = (int32_t)rec[4 * k + 1];
        const int64_t so = (int64_t)((uint64_t)rec[4 * k + 2] | ((uint64_t)rec[4 * k + 3] << 32));
        const char* base = BACK ? back_src : fd.src[0];
        if (!BACK && n_src > 1) base = fd.src[(ls >> LENSH_SHIFT) & (DC_MAX_SRC_SHARDS - 1)];
        e[k].st = st;
        e[k].en = st + (ls & LEN_MASK);
        e[k].ad = reinterpret_cast<int64_t>(base) + ((so - st) << lg);
    }

    constexpr int MAXU = 4;                                // chunks per lane: es of them are used
    uint32_t in_mask = 0, bnd_mask = 0;                    // bit u: chunk u is inside one slot / needs the element path
    gptr from[MAXU];
#pragma unroll
    for (int u = 0; u < MAXU; ++u) {
        from[u] = nullptr;
        if (u < es) {                                      // uniform
            const int32_t lo = u * tpi;                    // the instruction's first token inside the granule
            const int32_t c0 = lo + lane * tpc;            // my chunk's first token
            // scalar: the slot of the instruction's first token; does it cover all 64 chunks?
            int32_t s_en = INT32_MIN;
            int64_t s_ad = 0;
#pragma unroll
            for (int k = 0; k < REC_SLOTS; ++k)
                if (lo >= e[k].st) { s_en = e[k].en; s_ad = e[k].ad; }
            if (s_en >= lo + tpi && lo + tpi <= limit) {   // uniform: one slot, no search per lane
                in_mask |= 1u << u;
                from[u] = reinterpret_cast<gptr>(s_ad + ((int64_t)c0 << lg));
            } else {
                int32_t e_sel = INT32_MIN;
                int64_t a_sel = 0;
#pragma unroll
                for (int k = 0; k < REC_SLOTS; ++k)
                    if (c0 >= e[k].st) { e_sel = e[k].en; a_sel = e[k].ad; }
                const bool in = c0 + tpc <= e_sel && c0 + tpc <= limit;
                if (in) in_mask |= 1u << u;
                else if (c0 < limit) bnd_mask |= 1u << u;
                from[u] = reinterpret_cast<gptr>(a_sel + ((int64_t)c0 << lg));
            }
        }
    }
    // ---- chunks inside one slot: loads ----
    u32x4 v[MAXU];
    uint32_t x[MAXU];
#pragma unroll
    for (int u = 0; u < MAXU; ++u)
        if (in_mask & (1u << u)) load_chunk(from[u], v[u], x[u]);
    // ---- a chunk that touches a slot boundary, padding or the arena end is moved element by
    // element; the loads of a lane's first such chunk go out with the loads above, so a wave
    // with a sequence boundary in its granule (two waves in five) pays no second round trip
    const bool any_bnd = __ballot(bnd_mask != 0) != 0ull;                   // uniform
    BoundaryChunk bc;
    bc.ok = 0; bc.c0 = 0;
    if (any_bnd) {
        bc.c0 = (bnd_mask ? __builtin_ctz(bnd_mask) : 0) * tpi + lane * tpc;
        if (lg == 2) boundary_load<2>(e, bnd_mask != 0, limit, bc);
        else if (lg == 1) boundary_load<1>(e, bnd_mask != 0, limit, bc);
        else boundary_load<0>(e, bnd_mask != 0, limit, bc);
    }
    // ---- stores ----
#pragma unroll
    for (int u = 0; u < MAXU; ++u)
        if (in_mask & (1u << u)) {
            const uint32_t sh = (uint32_t)reinterpret_cast<uintptr_t>(from[u]) & 3u;
            gstore16(dst + (u * WAVE + lane) * 16, realign(v[u], x[u], sh));
        }
    if (!any_bnd) return;
    if (lg == 2) boundary_store<2>(dst, bc);
    else if (lg == 1) boundary_store<1>(dst, bc);
    else boundary_store<0>(dst, bc);
    // ---- further boundary chunks of the same lane (sequences shorter than a wave instruction) ----
    const uint32_t rest = bnd_mask & (bnd_mask - 1);
    if (__ballot(rest != 0) == 0ull) return;                                // uniform
#pragma unroll 1
    for (int u = 1; u < es; ++u) {
        const bool mine = (rest >> u) & 1u;
        if (__ballot(mine) == 0ull) continue;                               // uniform
        const int32_t c0 = u * tpi + lane * tpc;
        constexpr int EB = 4;                                               // elements in flight; divides 4, 8, 16
#pragma unroll 1
        for (int e0 = 0; e0 < tpc; e0 += EB) {
            uint32_t val[EB];
            bool ok[EB];
#pragma unroll
            for (int r = 0; r < EB; ++r) {
                const int32_t t = c0 + e0 + r;
                int32_t e_sel = INT32_MIN;
                int64_t a_sel = 0;
#pragma unroll
                for (int k = 0; k < REC_SLOTS; ++k)
                    if (t >= e[k].st) { e_sel = e[k].en; a_sel = e[k].ad; }
                ok[r] = mine && t < e_sel && t < limit;
                val[r] = 0;
                if (ok[r]) val[r] = load_elem(lg, reinterpret_cast<gptr>(a_sel + ((int64_t)t << lg)));
            }
#pragma unroll
            for (int r = 0; r < EB; ++r)
                if (ok[r]) store_elem(lg, dst + ((int64_t)(c0 + e0 + r) << lg), val[r]);
        }
    }
}

// ---------------------------------------------------------------- per-token advantage made on the way
// The advantage field of the training layout without its rollout-layout copy: the value of a
// token is its sequence's advantage where the sequence's mask byte is non-zero and +0.0f
// elsewhere (selection, as in the advantage stage), so the gather reads the 1-byte mask where
// it would read a 4-byte field.  These workgroups also move the mask field itself, from the
// bytes they have loaded anyway.
struct AdvSynth {
    const int32_t* perm;          // [N] slot -> sequence
    const float*   adv_seq;       // [N] advantage of every sequence
    float*         dst;           // float32 arena of the training layout
};
// It travels in the field table, in the entry behind the mask's (dst = the arena, src[0] = perm,
// src[1] = adv_seq), and is read from there by the workgroups that need it: as kernel arguments of
// their own the pointers would sit in scalar registers of every workgroup.
__device__ __forceinline__ AdvSynth adv_synth_of(const FieldDesc& fd) {
    AdvSynth s;
    s.perm = reinterpret_cast<const int32_t*>(fd.src[0]);
    s.adv_seq = reinterpret_cast<const float*>(fd.src[1]);
    s.dst = reinterpret_cast<float*>(fd.dst);
    return s;
}

__device__ __forceinline__ uint32_t sload1(const void* p) {
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wold-style-cast"
    return *(const DC_CONSTANT uint32_t*)p;
#pragma clang diagnostic pop
}

// Advantage bits of the output slots first .. first + REC_SLOTS - 1 (indices clamped into the
// arrays whatever perm holds).  Two batches of scalar loads: one round trip each.
__device__ __forceinline__ void slot_adv_scalar(const AdvSynth& s, int N, int first, uint32_t (&adv)[REC_SLOTS]) {
    uint32_t q[REC_SLOTS];
#pragma unroll
    for (int k = 0; k < REC_SLOTS; ++k) q[k] = sload1(s.perm + min(first + k, N - 1));
#pragma unroll
    for (int k = 0; k < REC_SLOTS; ++k) adv[k] = sload1(s.adv_seq + min(q[k], (uint32_t)(N - 1)));
}

// The two aligned words that hold the 4 mask bytes at byte address p (any alignment), and the
// output chunk of those 4 tokens.
__device__ __forceinline__ void load_mask4(gptr p, uint32_t& w0, uint32_t& w1) {
    const uintptr_t u = reinterpret_cast<uintptr_t>(p);
    gptr a4 = reinterpret_cast<gptr>(u & ~uintptr_t(3));
    w0 = gload4(a4);
    w1 = (u & 3) ? gload4(a4 + 4) : 0u;
}
__device__ __forceinline__ uint32_t mask4_of(uint32_t w0, uint32_t w1, gptr p) {
    return __builtin_amdgcn_alignbyte(w1, w0, (uint32_t)reinterpret_cast<uintptr_t>(p) & 3u);
}
__device__ __forceinline__ u32x4 select_adv4(uint32_t m, uint32_t adv) {
    u32x4 o;
    o.x = (m & 0x000000FFu) ? adv : 0u;
    o.y = (m & 0x0000FF00u) ? adv : 0u;
    o.z = (m & 0x00FF0000u) ? adv : 0u;
    o.w = (m & 0xFF000000u) ? adv : 0u;
    return o;
}

constexpr int ADV_TPC = 4;                    // tokens per 16-byte chunk of the float32 output
constexpr int ADV_TPI = WAVE * ADV_TPC;       // tokens one wave instruction covers

// The wave's granule of the advantage arena, slots from the granule's record, their advantage
// bits in adv[].  `mk` is the mask field.
__device__ __forceinline__ void adv_wave_sparse(const FieldDesc& mk, int n_src, const AdvSynth& s,
                                                const uint32_t (&adv)[REC_SLOTS], const u32x16& rec, int64_t wave_begin,
                                                int32_t limit) {
    const int lane = threadIdx.x & (WAVE - 1);
    gptr_w dst = reinterpret_cast<gptr_w>(reinterpret_cast<uintptr_t>(s.dst) + (wave_begin << 2));
    gptr_w mdst = reinterpret_cast<gptr_w>(reinterpret_cast<uintptr_t>(mk.dst) + wave_begin);

    const char* base[REC_SLOTS];                           // one batch of scalar loads
#pragma unroll
    for (int k = 0; k < REC_SLOTS; ++k)
        base[k] = n_src > 1 ? mk.src[((int32_t)rec[4 * k + 1] >> LENSH_SHIFT) & (DC_MAX_SRC_SHARDS - 1)] : mk.src[0];
    SlotS e[REC_SLOTS];                                    // ad: byte address of the granule's token 0 in the mask
#pragma unroll
    for (int k = 0; k < REC_SLOTS; ++k) {
        const int32_t st = (int32_t)rec[4 * k], ls = (int32_t)rec[4 * k + 1];
        const int64_t so = (int64_t)((uint64_t)rec[4 * k + 2] | ((uint64_t)rec[4 * k + 3] << 32));
        e[k].st = st;
        e[k].en = st + (ls & LEN_MASK);
        e[k].ad = reinterpret_cast<int64_t>(base[k]) + (so - st);
    }

    constexpr int NU = GATHER_GRAN / ADV_TPI;              // 4 chunks per lane
    uint32_t in_mask = 0, bnd_mask = 0;
    gptr from[NU];
    uint32_t av[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u) {
        const int32_t lo = u * ADV_TPI;
        const int32_t c0 = lo + lane * ADV_TPC;
        int32_t s_en = INT32_MIN;
        int64_t s_ad = 0;
        uint32_t s_av = 0;
#pragma unroll
        for (int k = 0; k < REC_SLOTS; ++k)
            if (lo >= e[k].st) { s_en = e[k].en; s_ad = e[k].ad; s_av = adv[k]; }
        if (s_en >= lo + ADV_TPI && lo + ADV_TPI <= limit) {       // uniform: one slot serves the instruction
            in_mask |= 1u << u;
            from[u] = reinterpret_cast<gptr>(s_ad + c0);
            av[u] = s_av;
        } else {
            int32_t e_sel = INT32_MIN;
            int64_t a_sel = 0;
            uint32_t v_sel = 0;
#pragma unroll
            for (int k = 0; k < REC_SLOTS; ++k)
                if (c0 >= e[k].st) { e_sel = e[k].en; a_sel = e[k].ad; v_sel = adv[k]; }
            const bool in = c0 + ADV_TPC <= e_sel && c0 + ADV_TPC <= limit;
            if (in) in_mask |= 1u << u;
            else if (c0 < limit) bnd_mask |= 1u << u;
            from[u] = reinterpret_cast<gptr>(a_sel + c0);
            av[u] = v_sel;
        }
    }
    uint32_t w0[NU], w1[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u)
        if (in_mask & (1u << u)) load_mask4(from[u], w0[u], w1[u]);
#pragma unroll
    for (int u = 0; u < NU; ++u)
        if (in_mask & (1u << u)) {
            const uint32_t m = mask4_of(w0[u], w1[u], from[u]);
            gstore16(dst + (u * WAVE + lane) * 16, select_adv4(m, av[u]));
            gstore4(mdst + (u * WAVE + lane) * 4, m);      // the mask's own move: the bytes are here already
        }
    // ---- chunks that touch a slot boundary, padding or the arena end: token by token ----
    if (__ballot(bnd_mask != 0) == 0ull) return;                             // uniform
#pragma unroll 1
    for (int u = 0; u < NU; ++u) {
        const bool mine = (bnd_mask >> u) & 1u;
        if (__ballot(mine) == 0ull) continue;                                // uniform
        const int32_t c0 = u * ADV_TPI + lane * ADV_TPC;
        uint32_t val[ADV_TPC], sel[ADV_TPC];
        bool ok[ADV_TPC];
#pragma unroll
        for (int r = 0; r < ADV_TPC; ++r) {
            const int32_t t = c0 + r;
            int32_t e_sel = INT32_MIN;
            int64_t a_sel = 0;
            sel[r] = 0;
#pragma unroll
            for (int k = 0; k < REC_SLOTS; ++k)
                if (t >= e[k].st) { e_sel = e[k].en; a_sel = e[k].ad; sel[r] = adv[k]; }
            ok[r] = mine && t < e_sel && t < limit;
            val[r] = 0;
            if (ok[r]) val[r] = load_elem(0, reinterpret_cast<gptr>(a_sel + t));
        }
#pragma unroll
        for (int r = 0; r < ADV_TPC; ++r)
            if (ok[r]) {
                store_elem(2, dst + ((int64_t)(c0 + r) << 2), val[r] ? sel[r] : 0u);
                store_elem(0, mdst + (c0 + r), val[r]);
            }
    }
}

// The same for a tile with many short sequences: slots staged in LDS (whole workgroup).
__device__ __forceinline__ void adv_tile_dense(const GatherArgs& a, SegLds& sg, uint32_t* sg_adv, const char* const* src,
                                               const AdvSynth& s, char* mask_dst, int seg_first, int seg_last,
                                               int64_t tile_begin, int32_t tile_len) {
    const int tid = threadIdx.x;
    const int N = a.n_seq;
    gptr_w dst = reinterpret_cast<gptr_w>(reinterpret_cast<uintptr_t>(s.dst) + (tile_begin << 2));
    gptr_w mdst = reinterpret_cast<gptr_w>(reinterpret_cast<uintptr_t>(mask_dst) + tile_begin);
    int seg_base = seg_first;
    int32_t pass_begin = 0;
    for (;;) {
        stage_slots(a, sg, src, 0, seg_base, seg_last, tile_begin);          // addresses in mask bytes
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int k = q * SEG_BATCH + tid;
            const int j = seg_base + k;
            if (q == 0 || tid < SEG_AHEAD) {
                uint32_t v = 0;
                if (j <= seg_last) {
                    const uint32_t sq = min((uint32_t)s.perm[j], (uint32_t)(N - 1));
                    v = __float_as_uint(s.adv_seq[sq]);
                }
                sg_adv[k] = v;
            }
        }
        __syncthreads();
        const int n_left = seg_last - seg_base + 1;
        const int n_all = min(n_left, NSEG);
        const bool more = n_left > SEG_BATCH && sg.start[SEG_BATCH] < tile_len;
        const int32_t pass_end = more ? sg.start[SEG_BATCH] : tile_len;
#pragma unroll 1
        for (int u = 0; u < GATHER_TILE_TOKENS / (GATHER_BLOCK * ADV_TPC); ++u) {
            const int32_t c0 = (tid + u * GATHER_BLOCK) * ADV_TPC;
            if (c0 < pass_begin || c0 >= pass_end) continue;
            int k = find_seg(sg.start, n_all, c0);
            if (k >= 0 && c0 + ADV_TPC <= sg.end[k] && c0 + ADV_TPC <= tile_len) {
                gptr ad = reinterpret_cast<gptr>(sg.addr[k] + c0);
                uint32_t w0, w1;
                load_mask4(ad, w0, w1);
                const uint32_t m = mask4_of(w0, w1, ad);
                gstore16(dst + (tid + u * GATHER_BLOCK) * 16, select_adv4(m, sg_adv[k]));
                gstore4(mdst + (tid + u * GATHER_BLOCK) * 4, m);
            } else {
                for (int r = 0; r < ADV_TPC; ++r) {
                    const int32_t tok = c0 + r;
                    if (tok >= tile_len) break;
                    while (k + 1 < n_all && sg.start[k + 1] <= tok) ++k;
                    if (k >= 0 && tok < sg.end[k]) {
                        const uint32_t m = load_elem(0, reinterpret_cast<gptr>(sg.addr[k] + tok));
                        store_elem(2, dst + ((int64_t)tok << 2), m ? sg_adv[k] : 0u);
                        store_elem(0, mdst + tok, m);
                    }
                }
            }
        }
        __syncthreads();
        if (!more) break;
        seg_base += SEG_BATCH;
        pass_begin = pass_end;
    }
}

// ---------------------------------------------------------------- the kernel
// The tile `tile` of carrier field fc.  BACK = false: the forward direction, fields as the
// table gives them.  BACK = true: the reverse direction, destination = the field's rollout
// buffer of segment seg, only source = its training arena.
template <bool BACK>
__device__ __forceinline__ void move_tile(const GatherArgs& a, const FieldTable& ft, uint32_t tile, uint32_t fc, int seg) {
    __shared__ SegLds sg;
    __shared__ const char* src[DC_MAX_SRC_SHARDS];
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / WAVE));
    const int N = a.n_seq;
    const int64_t tile_begin = (int64_t)tile * GATHER_TILE_TOKENS;
    const int64_t g0 = (int64_t)tile * GRAN_PER_TILE;

    // granule table of the tile: F[g] = first slot ending after granule g's first token; slots
    // F[g] .. F[g+1] are the ones that can reach into granule g.  The tables are padded, so the
    // entries of a whole tile (and one more) exist even for the last, partial tile.
    const u32x8 F = sload8(a.gran_first + g0);
    const u32x16 rec = sload16(a.gran_rec + g0 + w);
    const int first = (int)F[0];
    if (first < 0 || first >= N) return;                   // nothing reaches into this tile
    bool dense = false;
#pragma unroll
    for (int i = 0; i < GRAN_PER_TILE; ++i)
        dense = dense || ((int)F[i] < N && min((int)F[i + 1], N - 1) - (int)F[i] + 1 > REC_SLOTS);
    const int32_t limit = (int32_t)min((int64_t)GATHER_TILE_TOKENS, a.capacity - tile_begin);
    const int32_t wave_limit = min(limit - w * GATHER_GRAN, GATHER_GRAN);
    const int last = min(max((int)F[GRAN_PER_TILE], first), N - 1);

    for (uint32_t f = fc; f < a.n_carriers + a.n_riders; f = f < a.n_carriers ? a.n_carriers + f : f + a.n_carriers) {
        // f = fc, then the riders n_carriers + fc, n_carriers + fc + n_carriers, ...
        const FieldDesc& fd = ft.f[f];
        const int lg = fd.elem_bytes == 4 ? 2 : (fd.elem_bytes == 2 ? 1 : 0);
        char* back_dst = BACK ? const_cast<char*>(fd.src[seg]) : nullptr;
        const char* back_src = BACK ? fd.dst : nullptr;
        if (!dense) {
            if (wave_limit > 0)
                move_wave_sparse<BACK>(fd, ft.n_src, back_dst, back_src, lg, rec, tile_begin + w * GATHER_GRAN, wave_limit);
        } else {
            __syncthreads();                               // the previous field's readers of src[] and sg are done
            if (threadIdx.x < DC_MAX_SRC_SHARDS) src[threadIdx.x] = BACK ? back_src : fd.src[threadIdx.x];
            __syncthreads();
            move_tile_dense(a, sg, src, lg, BACK ? back_dst : fd.dst, first, last, tile_begin, limit);
        }
    }
}

// One workgroup per tile of GATHER_TILE_TOKENS tokens of one field, field-major.  Waves are short-lived on purpose: a wave that ends right
// after issuing its stores does not hold its slot until they are acknowledged, which a
// looping wave would (loads and stores retire through one in-order counter).
__global__ __launch_bounds__(GATHER_BLOCK) void gather_kernel(GatherArgs a, FieldTable ft) {
    // The grid walks the "carrier" fields, field after field (the 4-byte fields if there are
    // any, else every field).  Narrower fields ride along: rider r is moved by the waves of
    // carrier r mod n_carriers, right after their own data and from the same granule record.
    // A wave of a narrow field has only 1 or 2 KB in flight; as a workgroup of its own it
    // would hold a wave slot as long as a 4 KB one.
    move_tile<false>(a, ft, blockIdx.x % a.tiles, blockIdx.x / a.tiles, 0);
}

// The tile `tile` of the advantage arena and of the mask field.
__device__ __forceinline__ void adv_tile(const GatherArgs& a, const FieldTable& ft, uint32_t mask_field, uint32_t tile) {
    __shared__ SegLds sg;
    __shared__ uint32_t sg_adv[NSEG];
    __shared__ const char* src[DC_MAX_SRC_SHARDS];
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / WAVE));
    const int N = a.n_seq;
    const int64_t tile_begin = (int64_t)tile * GATHER_TILE_TOKENS;
    const int64_t g0 = (int64_t)tile * GRAN_PER_TILE;
    const u32x8 F = sload8(a.gran_first + g0);
    const u32x16 rec = sload16(a.gran_rec + g0 + w);
    const int first = (int)F[0];
    if (first < 0 || first >= N) return;
    bool dense = false;
#pragma unroll
    for (int i = 0; i < GRAN_PER_TILE; ++i)
        dense = dense || ((int)F[i] < N && min((int)F[i + 1], N - 1) - (int)F[i] + 1 > REC_SLOTS);
    const int32_t limit = (int32_t)min((int64_t)GATHER_TILE_TOKENS, a.capacity - tile_begin);
    const int32_t wave_limit = min(limit - w * GATHER_GRAN, GATHER_GRAN);
    const int last = min(max((int)F[GRAN_PER_TILE], first), N - 1);
    int wave_first = (int)F[0];
#pragma unroll
    for (int i = 1; i < GRAN_PER_TILE; ++i)
        if (w == i) wave_first = (int)F[i];

    const FieldDesc& mk = ft.f[mask_field];
    const AdvSynth s = adv_synth_of(ft.f[mask_field + 1]);
    if (!dense) {
        if (wave_limit > 0) {
            uint32_t adv[REC_SLOTS];
            slot_adv_scalar(s, N, wave_first, adv);
            adv_wave_sparse(mk, ft.n_src, s, adv, rec, tile_begin + w * GATHER_GRAN, wave_limit);
        }
    } else {
        if (threadIdx.x < DC_MAX_SRC_SHARDS) src[threadIdx.x] = mk.src[threadIdx.x];
        __syncthreads();
        adv_tile_dense(a, sg, sg_adv, src, s, mk.dst, first, last, tile_begin, limit);
    }
}

// gather_kernel with one more "carrier" behind the others: the advantage arena, made from the mask.
__global__ __launch_bounds__(GATHER_BLOCK) void gather_adv_kernel(GatherArgs a, FieldTable ft, uint32_t mask_field) {
    // The advantage tiles write four bytes for every byte they read; a run of them at the end of the
    // grid would be a pure write stream, which the memory serves more slowly than a mix.  They are
    // dealt in between the others instead: every (n_carriers + 1)-th workgroup takes one.
    const uint32_t per = a.n_carriers + 1;
    const uint32_t round = blockIdx.x / per, r = blockIdx.x % per;
    if (r == a.n_carriers) {
        adv_tile(a, ft, mask_field, (uint32_t)__builtin_amdgcn_readfirstlane((int)round));
    } else {
        const uint32_t idx = round * a.n_carriers + r;
        move_tile<false>(a, ft, (uint32_t)__builtin_amdgcn_readfirstlane((int)(idx % a.tiles)),
                         (uint32_t)__builtin_amdgcn_readfirstlane((int)(idx / a.tiles)), 0);
    }
}

// Reverse direction: the same grid over the tiles of all rollout buffers, one behind the other.
// a.dst_tok_off, a.slot_* and the granule tables arrive as the arrays of all segments; the
// workgroup narrows them to its segment's part.
__global__ __launch_bounds__(GATHER_BLOCK) void gather_back_kernel(GatherArgs a, FieldTable ft, BackSegs bs) {
    const uint32_t t = blockIdx.x % a.tiles;
    int seg = 0;
#pragma unroll
    for (int q = 0; q + 1 < DC_MAX_SRC_SHARDS; ++q) seg += t >= bs.tile_end[q] ? 1 : 0;   // t < tile_end[last]
    const uint32_t tile = t - (seg > 0 ? bs.tile_end[seg - 1] : 0u);
    const int first_seq = bs.first_seq[seg];
    a.n_seq = bs.n_seq[seg];
    a.capacity = bs.tokens[seg];
    a.dst_tok_off += first_seq + seg;
    a.slot_src_off += first_seq;
    a.slot_len += first_seq;
    a.slot_shard += first_seq;
    a.gran_first += bs.gran_base[seg];
    a.gran_rec += bs.gran_base[seg];
    move_tile<true>(a, ft, tile, blockIdx.x / a.tiles, seg);
}

// Field table with the 4-byte fields first (they carry, the others ride) and the grid's shape.
// skip >= 0: that field goes behind all others and neither carries nor rides (its place is returned).
static int order_fields(const FieldTable& ft, int64_t tiles, FieldTable* sorted, GatherArgs* a, int skip = -1) {
    *sorted = ft;
    int n = 0, n_wide = 0;
    for (int pass = 0; pass < 2; ++pass)
        for (int f = 0; f < ft.n_fields; ++f)
            if (f != skip && (ft.f[f].elem_bytes == 4) == (pass == 0)) {
                sorted->f[n++] = ft.f[f];
                if (pass == 0) n_wide = n;
            }
    const int n_moved = n;
    if (skip >= 0) sorted->f[n] = ft.f[skip];
    // riding pays when the carriers alone give the chip several rounds of workgroups; a small
    // batch needs every workgroup it can get
    const bool ride = n_wide > 0 && tiles * n_wide >= GATHER_RIDE_MIN_WGS;
    a->n_carriers = (uint32_t)(ride ? n_wide : n_moved);
    a->n_riders = (uint32_t)n_moved - a->n_carriers;
    a->tiles = (uint32_t)tiles;
    return n_moved;
}

hipError_t launch_gather(int32_t n_seq, const FieldTable& ft, int64_t dst_capacity,
                         const int64_t* d_dst_tok_off, const Workspace& ws, hipStream_t st,
                         hipEvent_t begins, hipEvent_t ends) {
    if (n_seq == 0 || ft.n_fields == 0 || dst_capacity == 0) return hipSuccess;
    GatherArgs a;
    a.n_seq = n_seq;
    a.capacity = dst_capacity;
    a.dst_tok_off = d_dst_tok_off;
    a.slot_src_off = ws.slot_src_off;
    a.slot_len = ws.slot_len;
    a.slot_shard = ws.slot_shard;
    a.gran_first = ws.gran_first;
    a.gran_rec = ws.gran_rec;
    const int64_t tiles = (dst_capacity + GATHER_TILE_TOKENS - 1) / GATHER_TILE_TOKENS;
    if (tiles * ft.n_fields > 0x7FFFFFFFLL || tiles * GRAN_PER_TILE + GRAN_PER_TILE + 1 > ws.n_gran)
        return hipErrorInvalidValue;
    FieldTable sorted;
    order_fields(ft, tiles, &sorted, &a);
    if (begins || ends)                                   // the dispatch itself carries the two events
        hipExtLaunchKernelGGL(gather_kernel, dim3((unsigned)(tiles * a.n_carriers)), dim3(GATHER_BLOCK), 0, st, begins, ends,
                              0, a, sorted);
    else
        hipLaunchKernelGGL(gather_kernel, dim3((unsigned)(tiles * a.n_carriers)), dim3(GATHER_BLOCK), 0, st, a, sorted);
    return hipGetLastError();
}

hipError_t launch_gather_advantage(int32_t n_seq, const FieldTable& ft, int mask_field, const int32_t* d_perm,
                                   const float* d_adv_seq, float* d_adv_tok_dst, int64_t dst_capacity,
                                   const int64_t* d_dst_tok_off, const Workspace& ws, hipStream_t st) {
    if (n_seq == 0 || dst_capacity == 0) return hipSuccess;
    if (mask_field < 0 || mask_field >= ft.n_fields || ft.f[mask_field].elem_bytes != 1) return hipErrorInvalidValue;
    GatherArgs a;
    a.n_seq = n_seq;
    a.capacity = dst_capacity;
    a.dst_tok_off = d_dst_tok_off;
    a.slot_src_off = ws.slot_src_off;
    a.slot_len = ws.slot_len;
    a.slot_shard = ws.slot_shard;
    a.gran_first = ws.gran_first;
    a.gran_rec = ws.gran_rec;
    const int64_t tiles = (dst_capacity + GATHER_TILE_TOKENS - 1) / GATHER_TILE_TOKENS;
    if (tiles * (ft.n_fields + 1) > 0x7FFFFFFFLL || tiles * GRAN_PER_TILE + GRAN_PER_TILE + 1 > ws.n_gran)
        return hipErrorInvalidValue;
    FieldTable sorted;
    const int at = order_fields(ft, tiles, &sorted, &a, mask_field);          // the mask's place; behind it:
    FieldDesc& syn = sorted.f[at + 1];
    syn.dst = reinterpret_cast<char*>(d_adv_tok_dst);
    syn.elem_bytes = 4;
    syn.src[0] = reinterpret_cast<const char*>(d_perm);
    syn.src[1] = reinterpret_cast<const char*>(d_adv_seq);
    hipLaunchKernelGGL(gather_adv_kernel, dim3((unsigned)(tiles * (a.n_carriers + 1))), dim3(GATHER_BLOCK), 0, st, a,
                       sorted, (uint32_t)at);
    return hipGetLastError();
}

hipError_t launch_gather_back(const BackSegs& bs, const FieldTable& ft, const ScatterWorkspace& ws, hipStream_t st) {
    const int64_t tiles = bs.tile_end[DC_MAX_SRC_SHARDS - 1];
    if (ft.n_fields == 0 || tiles == 0) return hipSuccess;
    if (tiles * ft.n_fields > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    for (int s = 0; s < DC_MAX_SRC_SHARDS; ++s) {           // every segment's tables hold its tiles plus the padding
        const int64_t seg_tiles = bs.tile_end[s] - (s > 0 ? bs.tile_end[s - 1] : 0u);
        if (seg_tiles > 0 && seg_tiles * GRAN_PER_TILE + GRAN_PER_TILE + 1 > bs.gran_base[s + 1] - bs.gran_base[s])
            return hipErrorInvalidValue;
    }
    if (bs.gran_base[DC_MAX_SRC_SHARDS] > ws.n_gran_all) return hipErrorInvalidValue;
    GatherArgs a;
    a.n_seq = 0;
    a.capacity = 0;
    a.dst_tok_off = ws.r_dst_off;
    a.slot_src_off = ws.r_src_off;
    a.slot_len = ws.r_len;
    a.slot_shard = ws.r_shard;
    a.gran_first = ws.gran_first;
    a.gran_rec = ws.gran_rec;
    FieldTable sorted;
    order_fields(ft, tiles, &sorted, &a);
    hipLaunchKernelGGL(gather_back_kernel, dim3((unsigned)(tiles * a.n_carriers)), dim3(GATHER_BLOCK), 0, st, a, sorted, bs);
    return hipGetLastError();
}

}  // namespace dc
