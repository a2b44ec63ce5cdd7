// Host planner: pool layout and lazy-allreduce buckets (Section 3.1), chunk
// table (Section 3.2), ring segments (Section 2.4), and the device copies of
// the tables the kernels index.
#include <algorithm>
#include <cmath>
#include <limits>
#include <new>

#include "gf_internal.h"

extern "C" const char *gf_status_string(gf_status s)
{
    switch (s) {
    case GF_OK: return "GF_OK";
    case GF_EINVAL: return "GF_EINVAL: invalid argument";
    case GF_ENOMEM: return "GF_ENOMEM: allocation failed";
    case GF_EHIP: return "GF_EHIP: HIP runtime error";
    case GF_ESTATE: return "GF_ESTATE: plan in the wrong state (tables not on the device, already uploaded, or on another device)";
    case GF_ELIMIT: return "GF_ELIMIT: the plan needs more scratch than gf_fuse_pack_static's fixed array holds";
    }
    return "unknown gf_status";
}

// Ring tables (Section 2.4).  A CSC plan reduces the packed buffer, whose length
// is only known at call time; a dense plan reduces each bucket, cut into one
// segment per rank of the ring (the masters, for a hierarchical allreduce).
static gf_status build_ring_tables(gf_plan *pl)
{
    pl->buckets.clear();
    pl->ring_blocks.clear();
    if (pl->chunk != 0) return GF_OK;
    const int64_t A = gf_wire_granule(pl->wire);
    for (size_t b = 0; b < pl->bucket_lo.size(); ++b) {
        gf_bucket_dev bd;
        bd.lo = pl->bucket_lo[b];
        bd.hi = pl->bucket_hi[b];
        bd.seg = gf_ring_segment_len(bd.hi - bd.lo, pl->ring_M, pl->wire);
        pl->buckets.push_back(bd);
        const int64_t Lb = bd.hi - bd.lo;
        for (int32_t s = 0; s < pl->ring_M; ++s) {
            const int64_t a = std::min<int64_t>(Lb, static_cast<int64_t>(s) * bd.seg);
            const int64_t e = std::min<int64_t>(Lb, a + bd.seg);
            const int64_t groups = (e - a + A - 1) / A;
            const int64_t blocks = (groups + GF_RING_GROUPS_PER_BLOCK - 1) / GF_RING_GROUPS_PER_BLOCK;
            for (int64_t i = 0; i < blocks; ++i) {
                gf_ring_block rb;
                rb.bucket = static_cast<int32_t>(b);
                rb.segment = s;
                rb.block_in_segment = static_cast<int32_t>(i);
                rb.pad_ = 0;
                pl->ring_blocks.push_back(rb);
            }
        }
    }
    if (pl->ring_blocks.size() > (size_t{1} << 30)) return GF_EINVAL;
    return GF_OK;
}

static gf_status build_plan(gf_plan *pl, const int64_t *numel, int32_t m, int64_t theta,
                            int32_t chunk, int32_t P, gf_wire wire)
{
    pl->m = m; pl->P = P; pl->chunk = chunk; pl->theta = theta; pl->wire = wire;
    pl->numel.assign(numel, numel + m);
    pl->off.resize(m);

    // Section 3.1: tensor m is generated first and sits at offset 0.
    int64_t run = 0;
    for (int32_t j = m - 1; j >= 0; --j) {
        if (numel[j] < 1 || run > std::numeric_limits<int64_t>::max() / 2 - numel[j]) return GF_EINVAL;
        pl->off[j] = run;
        run += numel[j];
    }
    pl->N = run;

    // Lazy allreduce (Section 3.1): a bucket that starts at pool offset `start` closes at the first
    // tensor end lying more than theta elements past it; what is left after tensor 1 is flushed.
    int64_t start = 0;
    for (int32_t j = m - 1; j >= 0; --j) {
        const int64_t end = pl->off[j] + numel[j];
        if (end - start > theta || j == 0) {
            pl->bucket_lo.push_back(start);
            pl->bucket_hi.push_back(end);
            start = end;
        }
    }

    // Work tiles: the chunks themselves for a CSC plan.
    pl->tile = chunk > 0 ? chunk : GF_DENSE_TILE;
    const int64_t n_tiles = (pl->N + pl->tile - 1) / pl->tile;
    if (n_tiles * static_cast<int64_t>(P) > (int64_t{1} << 30)) return GF_EINVAL;
    pl->n_tiles = static_cast<int32_t>(n_tiles);
    pl->n_chunks = chunk > 0 ? pl->n_tiles : 0;

    // Pieces of tensors per tile, pool order.
    pl->piece_start.assign(static_cast<size_t>(pl->n_tiles) + 1, 0);
    int64_t pos = 0;
    for (int32_t j = m - 1; j >= 0; --j) {
        int64_t left = numel[j], src = 0;
        while (left > 0) {
            const int64_t t = pos / pl->tile;
            const int64_t room = (t + 1) * pl->tile - pos;
            const int64_t len = std::min(left, room);
            gf_piece pc;
            pc.src_off = src;
            pc.tensor = j;
            pc.len = static_cast<int32_t>(len);
            pc.dst_rel = static_cast<int32_t>(pos - t * pl->tile);
            pc.pad_ = 0;
            pl->pieces.push_back(pc);
            pl->piece_start[static_cast<size_t>(t) + 1] += 1;
            pos += len; src += len; left -= len;
        }
    }
    for (int32_t t = 0; t < pl->n_tiles; ++t) pl->piece_start[t + 1] += pl->piece_start[t];

    // Sub-tiles of gf_fuse_pack that lie inside one tensor: where they start in it.
    const int32_t subs = gf_fuse_subs(pl);
    const int32_t sub_len = gf_fuse_sub_len(pl);
    pl->unit_src.assign(static_cast<size_t>(pl->n_tiles) * subs, gf_unit_src{0, -1, 0});
    for (int32_t t = 0; t < pl->n_tiles; ++t) {
        const int64_t tile_lo = static_cast<int64_t>(t) * pl->tile;
        const int64_t tile_len = std::min<int64_t>(pl->tile, pl->N - tile_lo);
        for (int32_t sb = 0; sb < subs; ++sb) {
            const int64_t lo = static_cast<int64_t>(sb) * sub_len;
            const int64_t hi = std::min<int64_t>(tile_len, lo + sub_len);
            if (hi <= lo) continue;
            for (int32_t i = pl->piece_start[t]; i < pl->piece_start[t + 1]; ++i) {
                const gf_piece &pc = pl->pieces[i];
                if (pc.dst_rel <= lo && pc.dst_rel + pc.len >= hi) {
                    gf_unit_src &us = pl->unit_src[static_cast<size_t>(t) * subs + sb];
                    us.tensor = pc.tensor;
                    us.src_off = pc.src_off + (lo - pc.dst_rel);
                    break;
                }
            }
        }
    }

    pl->ring_M = P;
    return build_ring_tables(pl);
}

extern "C" gf_status gf_plan_create(gf_plan **out, const int64_t *tensor_numel, int32_t m,
                                    int64_t theta_elems, int32_t chunk_elems, int32_t P, gf_wire wire)
{
    if (!out) return GF_EINVAL;
    *out = nullptr;
    if (!tensor_numel || m < 1 || theta_elems < 0 || chunk_elems < 0 || P < 1 || P > 4096) return GF_EINVAL;
    if (chunk_elems > (1 << 28)) return GF_EINVAL;      // a chunk's byte offsets must fit 32 bits
    if (wire != GF_WIRE_F16 && wire != GF_WIRE_F32) return GF_EINVAL;
    gf_plan *pl = new (std::nothrow) gf_plan;
    if (!pl) return GF_ENOMEM;
    gf_status st;
    try {
        st = build_plan(pl, tensor_numel, m, theta_elems, chunk_elems, P, wire);
    } catch (const std::bad_alloc &) {
        st = GF_ENOMEM;
    }
    if (st != GF_OK) { delete pl; return st; }
    *out = pl;
    return GF_OK;
}

template <typename T>
static gf_status upload(T **dst, const std::vector<T> &src)
{
    *dst = nullptr;
    if (src.empty()) return GF_OK;
    if (hipMalloc(reinterpret_cast<void **>(dst), src.size() * sizeof(T)) != hipSuccess) {
        (void)hipGetLastError();
        *dst = nullptr;
        return GF_ENOMEM;
    }
    GF_HIP_TRY(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice));
    return GF_OK;
}

static void free_device(gf_plan *pl)
{
    if (pl->d_piece_start) (void)hipFree(pl->d_piece_start);
    if (pl->d_pieces) (void)hipFree(pl->d_pieces);
    if (pl->d_unit_src) (void)hipFree(pl->d_unit_src);
    if (pl->d_buckets) (void)hipFree(pl->d_buckets);
    if (pl->d_ring_blocks) (void)hipFree(pl->d_ring_blocks);
    pl->d_piece_start = nullptr; pl->d_pieces = nullptr; pl->d_unit_src = nullptr;
    pl->d_buckets = nullptr; pl->d_ring_blocks = nullptr;
    pl->on_device = false;
}

extern "C" gf_status gf_plan_to_device(gf_plan *pl)
{
    if (!pl) return GF_EINVAL;
    if (pl->on_device) return GF_OK;
    GF_HIP_TRY(hipGetDevice(&pl->device));
    gf_status st = upload(&pl->d_piece_start, pl->piece_start);
    if (st == GF_OK) st = upload(&pl->d_pieces, pl->pieces);
    if (st == GF_OK) st = upload(&pl->d_unit_src, pl->unit_src);
    if (st == GF_OK) st = upload(&pl->d_buckets, pl->buckets);
    if (st == GF_OK) st = upload(&pl->d_ring_blocks, pl->ring_blocks);
    if (st != GF_OK) { free_device(pl); return st; }
    pl->on_device = true;
    return GF_OK;
}

extern "C" void gf_plan_destroy(gf_plan *pl)
{
    if (!pl) return;
    if (pl->on_device) free_device(pl);
    delete pl;
}

extern "C" gf_status gf_plan_info(const gf_plan *pl, int64_t *N, int32_t *n_chunks, int32_t *n_buckets)
{
    if (!pl) return GF_EINVAL;
    if (N) *N = pl->N;
    if (n_chunks) *n_chunks = pl->n_chunks;
    if (n_buckets) *n_buckets = static_cast<int32_t>(pl->bucket_lo.size());
    return GF_OK;
}

extern "C" gf_status gf_plan_layout(const gf_plan *pl, int64_t *tensor_off, int64_t *bucket_lo,
                                    int64_t *bucket_hi)
{
    if (!pl) return GF_EINVAL;
    if (tensor_off) std::copy(pl->off.begin(), pl->off.end(), tensor_off);
    if (bucket_lo) std::copy(pl->bucket_lo.begin(), pl->bucket_lo.end(), bucket_lo);
    if (bucket_hi) std::copy(pl->bucket_hi.begin(), pl->bucket_hi.end(), bucket_hi);
    return GF_OK;
}

extern "C" int64_t gf_plan_ring_segment(const gf_plan *pl, int64_t L)
{
    if (!pl || L < 0) return -1;
    return gf_ring_segment_len(L, pl->ring_M, pl->wire);
}

extern "C" int32_t gf_plan_tiles(const gf_plan *pl) { return pl ? pl->n_tiles : -1; }

extern "C" int32_t gf_plan_tile_pieces(const gf_plan *pl, int32_t tile, int32_t cap,
                                       int32_t *tensor, int64_t *src_off, int32_t *len)
{
    if (!pl || tile < 0 || tile >= pl->n_tiles || cap < 0) return -1;
    const int32_t a = pl->piece_start[tile], b = pl->piece_start[tile + 1];
    for (int32_t i = a; i < b && i - a < cap; ++i) {
        if (tensor) tensor[i - a] = pl->pieces[i].tensor;
        if (src_off) src_off[i - a] = pl->pieces[i].src_off;
        if (len) len[i - a] = pl->pieces[i].len;
    }
    return b - a;
}

extern "C" size_t gf_plan_workspace_bytes(const gf_plan *pl)
{
    if (!pl) return 0;
    return gf_ws_total_bytes(pl);
}

// Warm-up dense training (Section 3.2): the sparsity ratio ramps linearly from
// zero to its final value over the warm-up iterations.
extern "C" int32_t gf_plan_warmup_k(const gf_plan *pl, double final_density, int64_t iteration,
                                    int64_t warmup_iterations)
{
    if (!pl || pl->chunk == 0 || !(final_density > 0.0) || final_density > 1.0 || iteration < 0 ||
        warmup_iterations < 0)
        return -1;
    double s = 1.0 - final_density;
    if (warmup_iterations > 0) {
        const int64_t t = iteration < warmup_iterations ? iteration : warmup_iterations;
        s = s * static_cast<double>(t) / static_cast<double>(warmup_iterations);
    }
    const double want = std::ceil((1.0 - s) * static_cast<double>(pl->n_chunks) - 1e-9);
    int64_t k = static_cast<int64_t>(want);
    if (k < 1) k = 1;
    if (k > pl->n_chunks) k = pl->n_chunks;
    return static_cast<int32_t>(k);
}

// Section 3.1: the pool may hold FP16 gradients (mixed-precision backward).
extern "C" gf_status gf_plan_set_grad_type(gf_plan *pl, gf_wire type)
{
    if (!pl || (type != GF_WIRE_F16 && type != GF_WIRE_F32)) return GF_EINVAL;
    pl->grad = type;
    return GF_OK;
}

// Section 2.4, hierarchical allreduce: M groups of P / M consecutive ranks, the
// lowest rank of each group its master.  M = P (or 0) is the flat ring.
extern "C" gf_status gf_plan_set_reduce_groups(gf_plan *pl, int32_t M)
{
    if (!pl || M < 0 || M > pl->P) return GF_EINVAL;
    if (M == 0) M = pl->P;
    if (pl->P % M != 0) return GF_EINVAL;
    if (pl->on_device) return GF_ESTATE;       // the ring tables already went to the device
    if (M == pl->ring_M) return GF_OK;
    pl->ring_M = M;
    try {
        return build_ring_tables(pl);
    } catch (const std::bad_alloc &) {
        return GF_ENOMEM;
    }
}
