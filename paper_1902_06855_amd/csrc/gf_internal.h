// Internal definitions shared by the library's translation units (not part of
// the C ABI).
#ifndef GF_INTERNAL_H
#define GF_INTERNAL_H

#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "gf.h"

// Work tile of a dense-only plan, in pool elements.  Any multiple of 8 works;
// 8192 elements = 32 KB of fp32 per worker per tile keeps >25k workgroups in
// flight on the ResNet-50-sized pool while amortising the per-tile set-up.
constexpr int32_t GF_DENSE_TILE = 8192;

// gf_fuse_pack cuts tiles longer than this into sub-tiles of this many elements
// (a multiple of 4), one workgroup each.
constexpr int32_t GF_FUSE_SUB = 8192;

// One contiguous run of a tensor inside a tile (pool order).
struct gf_piece {
    int64_t src_off;   // first element inside the tensor
    int32_t tensor;    // 0-based ID index
    int32_t len;       // elements
    int32_t dst_rel;   // offset of the run from the tile's first pool element
    int32_t pad_;
};
static_assert(sizeof(gf_piece) == 24, "piece record layout");

// Where the gradients of one sub-tile of gf_fuse_pack live when they lie inside a
// single tensor (the common case): saves the walk through the piece table.
struct gf_unit_src {
    int64_t src_off;   // first element inside the tensor
    int32_t tensor;    // 0-based ID index, or -1: several tensors meet in this sub-tile
    int32_t pad_;
};
static_assert(sizeof(gf_unit_src) == 16, "unit source record layout");

// Ring work item of a dense plan: one workgroup's share of one segment of one
// bucket.  (A workgroup never straddles segments, so the fold's starting
// worker is uniform across it.)
struct gf_ring_block {
    int32_t bucket;
    int32_t segment;
    int32_t block_in_segment;
    int32_t pad_;
};

struct gf_bucket_dev {
    int64_t lo, hi;    // pool element range
    int64_t seg;       // ring segment length, elements
};

struct gf_plan {
    // host
    int32_t m = 0, P = 0, chunk = 0, tile = 0, n_tiles = 0, n_chunks = 0;
    int64_t N = 0, theta = 0;
    gf_wire wire = GF_WIRE_F16;
    gf_wire grad = GF_WIRE_F32;                  // element type of the gradients handed to gf_fuse_pack
    int32_t ring_M = 0;                          // ranks in the ring (P, or the masters of a hierarchical allreduce)
    std::vector<int64_t> numel, off;             // ID order
    std::vector<int64_t> bucket_lo, bucket_hi;   // generation order
    std::vector<int32_t> piece_start;            // [n_tiles + 1]
    std::vector<gf_piece> pieces;
    std::vector<gf_unit_src> unit_src;           // [n_tiles * gf_fuse_subs]
    std::vector<gf_bucket_dev> buckets;
    std::vector<gf_ring_block> ring_blocks;      // dense plans only
    // device (valid once on_device)
    bool on_device = false;
    int device = -1;
    int32_t *d_piece_start = nullptr;
    gf_piece *d_pieces = nullptr;
    gf_unit_src *d_unit_src = nullptr;
    gf_bucket_dev *d_buckets = nullptr;
    gf_ring_block *d_ring_blocks = nullptr;
};

// Elements per 16 bytes of the wire type: the ring's segment granule.
inline int64_t gf_wire_granule(gf_wire w) { return w == GF_WIRE_F16 ? 8 : 4; }
inline int64_t gf_wire_bytes(gf_wire w) { return w == GF_WIRE_F16 ? 2 : 4; }

inline int64_t gf_ring_segment_len(int64_t L, int32_t P, gf_wire w)
{
    const int64_t A = gf_wire_granule(w);
    const int64_t per = (L + P - 1) / P;
    return (per + A - 1) / A * A;
}

// Elements per full lazy-allreduce bucket of a CSC plan's packed buffer: the
// bucket closes after the chunk that makes the waited size exceed theta.
inline int64_t gf_csc_bucket_span(const gf_plan *p)
{
    int64_t q = p->theta / p->chunk + 1;
    if (q > p->n_chunks) q = p->n_chunks;
    return q * p->chunk;
}

// Threads per workgroup of the streaming kernels, and 16-byte groups each ring
// workgroup covers.
constexpr int GF_BLOCK = 256;
constexpr int GF_RING_GROUPS_PER_BLOCK = 512;   // = threads of a ring workgroup

#define GF_HIP_TRY(expr)                        \
    do {                                        \
        if ((expr) != hipSuccess) {             \
            (void)hipGetLastError();            \
            return GF_EHIP;                     \
        }                                       \
    } while (0)

// Compute calls run on the device the plan's tables were uploaded to.
#define GF_CHECK_DEVICE(pl)                                         \
    do {                                                            \
        int cur_ = -1;                                              \
        GF_HIP_TRY(hipGetDevice(&cur_));                            \
        if (cur_ != (pl)->device) return GF_ESTATE;                 \
    } while (0)

#define GF_LAUNCH_CHECK()                       \
    do {                                        \
        if (hipGetLastError() != hipSuccess)    \
            return GF_EHIP;                     \
    } while (0)

// Workspace layout (bytes from the 256-byte aligned base).
inline size_t gf_ws_slotmap_off() { return 0; }
inline size_t gf_ws_slotmap_bytes(const gf_plan *p)
{
    return (static_cast<size_t>(p->n_chunks) * sizeof(int32_t) + 255) / 256 * 256;
}
inline size_t gf_ws_scores_off(const gf_plan *p) { return gf_ws_slotmap_bytes(p); }
inline size_t gf_ws_scores_bytes(const gf_plan *p)
{
    return (static_cast<size_t>(p->n_chunks) * sizeof(float) + 255) / 256 * 256;
}
// Sub-tiles per tile in gf_fuse_pack, and the partial chunk norms they leave
// behind (one double per worker, chunk and sub-tile) when there are several, or
// when the caller leaves the norms in the workspace for gf_chunk_score_select.
inline int32_t gf_fuse_subs(const gf_plan *p)
{
    return p->tile <= GF_FUSE_SUB ? 1 : (p->tile + GF_FUSE_SUB - 1) / GF_FUSE_SUB;
}
// Sub-tile length.  Sub-tiles of exactly GF_FUSE_SUB elements (the last one of a tile takes what
// is left) measured faster than equal parts: their starts stay 128-byte aligned within the tile.
inline int32_t gf_fuse_sub_len(const gf_plan *p) { return p->tile < GF_FUSE_SUB ? p->tile : GF_FUSE_SUB; }
inline size_t gf_ws_l1part_off(const gf_plan *p) { return gf_ws_slotmap_bytes(p) + gf_ws_scores_bytes(p); }
inline size_t gf_ws_l1part_bytes(const gf_plan *p)
{
    if (p->chunk == 0) return 0;
    return (static_cast<size_t>(p->P) * p->n_chunks * gf_fuse_subs(p) * sizeof(double) + 255) / 256 * 256;
}
inline size_t gf_ws_total_bytes(const gf_plan *p)
{
    return gf_ws_slotmap_bytes(p) + gf_ws_scores_bytes(p) + gf_ws_l1part_bytes(p) + 256;
}

#endif  // GF_INTERNAL_H
