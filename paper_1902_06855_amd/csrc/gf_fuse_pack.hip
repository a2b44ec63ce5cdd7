// gf_fuse_pack: lazy-allreduce fusion folded into the read (Section 3.1), the
// allreduce-preprocess step of Algorithm 1 (g + hg, then hg = 0 or
// momentum * g), per-chunk L1 norms (Section 3.2) and the fp32 -> wire cast
// with loss scaling (Section 2.5), as one HBM-streaming pass per worker tile.
//
// One workgroup handles one (worker, tile) pair; a tile is a chunk of a CSC
// plan or a fixed slice of the pool of a dense plan.  Whether the tile is sent
// is uniform across the workgroup, so each case runs its own straight-line
// inner loop of 128-bit loads and stores with several loads in flight.  With
// scattered per-tensor gradients a tile may be made of pieces of several
// tensors; their addresses are put in a small LDS table so that the tile is
// still swept as one run.
#include <type_traits>

#include "gf_device.h"

namespace {

enum : int {
    F_G = 1,          // read gradients
    F_RES = 2,        // read the historical gradient
    F_SEND = 4,       // write wire(acc * S)
    F_KEEP = 8,       // hg <- mu * acc
    F_ZERO = 16,      // hg <- +0
    F_L1 = 32         // accumulate |acc|
};

enum : int { MODE_ACCUM = 0, MODE_FUSED = 1, MODE_DENSE = 2, MODE_PACK = 3, MODE_SCALE = 4 };

struct FuseArgs {
    const void *const *tab;      // gradient pointer table (grads or pools)
    int32_t tab_stride;          // m for grads, 1 for pools
    int32_t use_pieces;          // 1: gather through the piece table
    float *const *residual;
    void *const *sendbuf;
    const int32_t *slotmap;      // [n_tiles] rank among the selected chunks or -1; NULL: rank = tile
    const int32_t *sel_idx;      // MODE_PACK: tiles to visit; NULL: all
    float *chunk_l1;
    const int32_t *piece_start;
    const gf_piece *pieces;
    int64_t N;
    int32_t tile, n_tiles, units; // units: work items per worker
    float S, mu;
};

template <int F, typename W>
__device__ __forceinline__ void elem4(const gf_f32x4 g, const gf_f32x4 r, gf_f32x4 &res_out,
                                      typename gf_wire4<W>::type &snd_out, float S, float mu, double &l1)
{
    float a0, a1, a2, a3;
    if constexpr ((F & F_G) && (F & F_RES)) { a0 = g.x + r.x; a1 = g.y + r.y; a2 = g.z + r.z; a3 = g.w + r.w; }
    else if constexpr (F & F_G) { a0 = g.x; a1 = g.y; a2 = g.z; a3 = g.w; }
    else { a0 = r.x; a1 = r.y; a2 = r.z; a3 = r.w; }
    if constexpr (F & F_L1) {
        l1 += static_cast<double>(fabsf(a0));
        l1 += static_cast<double>(fabsf(a1));
        l1 += static_cast<double>(fabsf(a2));
        l1 += static_cast<double>(fabsf(a3));
    }
    if constexpr (F & F_SEND)
        snd_out = gf_pack4(gf_to_wire<W>(a0 * S), gf_to_wire<W>(a1 * S), gf_to_wire<W>(a2 * S), gf_to_wire<W>(a3 * S));
    if constexpr (F & F_KEEP) res_out = gf_pack4(mu * a0, mu * a1, mu * a2, mu * a3);
    if constexpr (F & F_ZERO) res_out = gf_pack4(0.f, 0.f, 0.f, 0.f);
}

// Source of the gradients of one tile.
//   direct: one contiguous run starting at `base` (pool input, or a tile that
//           lies inside a single tensor);
//   flat:   several tensor pieces; piece i covers tile offsets
//           [end[i-1], end[i]) and element x of the tile is at ptr[i][x].
// In both cases `at(x)` is only evaluated for x inside the tile.
// GT is the gradients' element type: float, or uint16_t for fp16 gradients
// (Section 3.1: the pool holds FP32 or FP16 gradients).
template <typename GT>
struct GradSrc {
    const GT *base;
    const GT *const *ptr;         // LDS
    const int *end;               // LDS
    int n;                        // pieces (0 = direct)
    __device__ __forceinline__ const GT *at(int x) const
    {
        if (n == 0) return base + x;
        int i = 0;
        while (i + 1 < n && x >= end[i]) ++i;
        return ptr[i] + x;
    }
};

// One tile (or one contiguous piece of it) of `len` elements.  res / snd are
// already offset to its first element; unused pointers are null.  Gradients
// and the historical gradient are touched exactly once per iteration, so they
// go around the caches (nontemporal); the send buffer is read back by the ring
// kernel right away and stays cacheable.
template <int F, typename W, typename GT, int NT, int U>
__device__ __forceinline__ void run(const GradSrc<GT> &src, float *res_, W *snd_, int len, bool vec,
                                    float S, float mu, double &l1)
{
    using G4 = typename gf_wire4<GT>::type;                // four gradients as stored
    GF_GLOBAL float *__restrict__ res = gf_global(res_);
    GF_GLOBAL W *__restrict__ snd = gf_global(snd_);
    using W4 = typename gf_wire4<W>::type;
    constexpr bool WRITES_RES = (F & (F_KEEP | F_ZERO)) != 0;
    if constexpr ((F & F_RES) || WRITES_RES) vec = vec && gf_aligned(res, 16);
    if constexpr (F & F_SEND) vec = vec && gf_aligned(snd, sizeof(W4));
    const int nvec = vec ? (len >> 2) : 0;
    auto g4 = [&](int v) { return reinterpret_cast<const GF_GLOBAL G4 *>(gf_global(src.at(v << 2))); };
    auto widen = [](G4 x) { float a, b, c, d; gf_unpack4(x, a, b, c, d); return gf_pack4(a, b, c, d); };

    // 128-bit sweep.  A direct source goes through buffer descriptors (one per stream, made
    // for exactly this run); a tile pieced together from several tensors reads its gradients
    // through per-lane global addresses instead.
    constexpr int WB = static_cast<int>(sizeof(W4));      // bytes of four wire elements
    const uint32_t run_bytes = static_cast<uint32_t>(len) * 4u;
    constexpr int GB = static_cast<int>(sizeof(G4));      // bytes of four gradients
    const __amdgpu_buffer_rsrc_t gb = gf_make_buf(gf_global(src.base), (F & F_G) && src.n == 0
                                                  ? static_cast<uint32_t>(len) * sizeof(GT) : 0u);
    const __amdgpu_buffer_rsrc_t rb = gf_make_buf(res, ((F & F_RES) || WRITES_RES) ? run_bytes : 0u);
    const __amdgpu_buffer_rsrc_t sb = gf_make_buf(snd, (F & F_SEND) ? static_cast<uint32_t>(len) * sizeof(W) : 0u);
    auto sweep = [&](auto direct_tag) {
        constexpr bool DIRECT = decltype(direct_tag)::value;
        auto load_g = [&](int v) {
            if constexpr (DIRECT) {
                if constexpr (sizeof(GT) == 4) return gf_buf_ld128<GF_AUX_STREAM>(gb, v * GB);
                else return widen(gf_buf_ld64u<GF_AUX_STREAM>(gb, v * GB));
            } else {
                return widen(gf_ld_stream(g4(v)));
            }
        };
        int v = threadIdx.x;
        for (; v + (U - 1) * NT < nvec; v += U * NT) {
            gf_f32x4 gg[U], rr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if constexpr (F & F_G) gg[u] = load_g(v + u * NT);
                if constexpr (F & F_RES) rr[u] = gf_buf_ld128<GF_AUX_STREAM>(rb, (v + u * NT) * 16);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                gf_f32x4 ro; W4 so;
                elem4<F, W>(gg[u], rr[u], ro, so, S, mu, l1);
                if constexpr (WRITES_RES) gf_buf_st<GF_AUX_STREAM>(ro, rb, (v + u * NT) * 16);
                if constexpr (F & F_SEND) gf_buf_st<GF_AUX_CACHED>(so, sb, (v + u * NT) * WB);
            }
        }
        for (; v < nvec; v += NT) {
            gf_f32x4 gg = {}, rr = {}, ro; W4 so;
            if constexpr (F & F_G) gg = load_g(v);
            if constexpr (F & F_RES) rr = gf_buf_ld128<GF_AUX_STREAM>(rb, v * 16);
            elem4<F, W>(gg, rr, ro, so, S, mu, l1);
            if constexpr (WRITES_RES) gf_buf_st<GF_AUX_STREAM>(ro, rb, v * 16);
            if constexpr (F & F_SEND) gf_buf_st<GF_AUX_CACHED>(so, sb, v * WB);
        }
    };
    if (src.n == 0) sweep(std::true_type{});
    else sweep(std::false_type{});
    for (int i = (nvec << 2) + threadIdx.x; i < len; i += NT) {   // unaligned data or ragged tail
        float a;
        if constexpr ((F & F_G) && (F & F_RES)) a = gf_from_wire<GT>(*gf_global(src.at(i))) + res[i];
        else if constexpr (F & F_G) a = gf_from_wire<GT>(*gf_global(src.at(i)));
        else a = res[i];
        if constexpr (F & F_L1) l1 += static_cast<double>(fabsf(a));
        if constexpr (F & F_SEND) snd[i] = gf_to_wire<W>(a * S);
        if constexpr (F & F_KEEP) res[i] = mu * a;
        if constexpr (F & F_ZERO) res[i] = 0.f;
    }
}

constexpr int MAX_FLAT_PIECES = 64;   // more pieces than this in one tile are walked one by one

template <int F, typename W, typename GT, int NT, int U>
__device__ __forceinline__ void tile_body(const FuseArgs &a, int p, int tile, int64_t slot, double &l1)
{
    constexpr unsigned GALIGN = 4 * sizeof(GT);            // alignment the vector path needs
    const int64_t tile_lo = static_cast<int64_t>(tile) * a.tile;
    const int64_t left = a.N - tile_lo;
    const int tile_len = left < a.tile ? static_cast<int>(left) : a.tile;
    constexpr bool USES_RES = (F & (F_RES | F_KEEP | F_ZERO)) != 0;
    float *res = USES_RES ? a.residual[p] + tile_lo : nullptr;
    W *snd = (F & F_SEND) ? static_cast<W *>(a.sendbuf[p]) + slot * a.tile : nullptr;
    GradSrc<GT> src{nullptr, nullptr, nullptr, 0};
    if constexpr ((F & F_G) == 0) {
        run<F, W, GT, NT, U>(src, res, snd, tile_len, true, a.S, a.mu, l1);
        return;
    }
    if (!a.use_pieces) {
        src.base = static_cast<const GT *>(a.tab[p]) + tile_lo;
        run<F, W, GT, NT, U>(src, res, snd, tile_len, gf_aligned(src.base, GALIGN), a.S, a.mu, l1);
        return;
    }
    const int ps = a.piece_start[tile], np = a.piece_start[tile + 1] - ps;
    const GT *const *tab = reinterpret_cast<const GT *const *>(a.tab) + static_cast<int64_t>(p) * a.tab_stride;
    if (np == 1) {
        const gf_piece pc = a.pieces[ps];
        src.base = tab[pc.tensor] + pc.src_off;
        run<F, W, GT, NT, U>(src, res, snd, tile_len, gf_aligned(src.base, GALIGN), a.S, a.mu, l1);
        return;
    }
    if (np <= MAX_FLAT_PIECES) {
        // Several tensors meet in this tile: publish where each piece lives, then
        // sweep the tile as if it were one run.
        __shared__ const GT *s_ptr[MAX_FLAT_PIECES];
        __shared__ int s_end[MAX_FLAT_PIECES];
        int misaligned = 0;
        if (static_cast<int>(threadIdx.x) < np) {
            const gf_piece pc = a.pieces[ps + threadIdx.x];
            const GT *q = tab[pc.tensor] + pc.src_off;
            s_ptr[threadIdx.x] = q - pc.dst_rel;
            s_end[threadIdx.x] = pc.dst_rel + pc.len;
            misaligned = !gf_aligned(q, GALIGN) || (pc.dst_rel & 3);
        }
        const bool vec = !__syncthreads_or(misaligned);
        src.ptr = s_ptr; src.end = s_end; src.n = np;
        run<F, W, GT, NT, U>(src, res, snd, tile_len, vec, a.S, a.mu, l1);
        __syncthreads();                       // the table is reused by the next caller
        return;
    }
    for (int i = ps; i < ps + np; ++i) {
        const gf_piece pc = a.pieces[i];
        src.base = tab[pc.tensor] + pc.src_off;
        run<F, W, GT, NT, U>(src, USES_RES ? res + pc.dst_rel : nullptr, (F & F_SEND) ? snd + pc.dst_rel : nullptr,
                         pc.len, gf_aligned(src.base, GALIGN), a.S, a.mu, l1);
    }
}

// One workgroup per (worker, tile).  WPE caps the wavefronts resident per SIMD
// (0 = no cap): fewer resident workgroups mean fewer DRAM pages open at once,
// which the in-place read-read-write stream of short tiles rewards.
template <int MODE, typename W, typename GT, int NT, int U, int WPE>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WPE ? WPE : 1, WPE ? WPE : 8)))
void k_fuse(const FuseArgs a)
{
    const int p = blockIdx.x / a.units;
    const int u = blockIdx.x - p * a.units;
    int tile = u;
    int64_t slot = u;
    if constexpr (MODE == MODE_PACK) {
        if (a.sel_idx) tile = a.sel_idx[u];
    } else if constexpr (MODE == MODE_FUSED || MODE == MODE_SCALE) {
        if (a.slotmap) slot = a.slotmap[tile];
    }
    double l1 = 0.0;
    if constexpr (MODE == MODE_ACCUM) tile_body<F_G | F_RES | F_KEEP | F_L1, W, GT, NT, U>(a, p, tile, 0, l1);   // mu = 1 here
    if constexpr (MODE == MODE_FUSED) {
        if (slot >= 0) tile_body<F_G | F_RES | F_SEND | F_ZERO | F_L1, W, GT, NT, U>(a, p, tile, slot, l1);
        else tile_body<F_G | F_RES | F_KEEP | F_L1, W, GT, NT, U>(a, p, tile, 0, l1);
    }
    if constexpr (MODE == MODE_DENSE) tile_body<F_G | F_SEND, W, GT, NT, U>(a, p, tile, slot, l1);
    if constexpr (MODE == MODE_PACK) tile_body<F_RES | F_SEND | F_ZERO, W, GT, NT, U>(a, p, tile, slot, l1);
    if constexpr (MODE == MODE_SCALE) {
        if (slot < 0) tile_body<F_RES | F_KEEP, W, GT, NT, U>(a, p, tile, 0, l1);
    }
    if constexpr (MODE == MODE_ACCUM || MODE == MODE_FUSED) {
        const double s = gf_block_sum<NT>(l1);
        if (a.chunk_l1 && threadIdx.x == 0)
            a.chunk_l1[static_cast<int64_t>(p) * a.n_tiles + tile] = static_cast<float>(s);
    }
}

// slotmap[c] = rank of chunk c in the ascending selection, or -1.
__global__ __launch_bounds__(GF_BLOCK) void k_slotmap(const int32_t *__restrict__ sel, int32_t k,
                                                      int32_t n_chunks, int32_t *__restrict__ slotmap)
{
    const int c = blockIdx.x * GF_BLOCK + threadIdx.x;
    if (c >= n_chunks) return;
    int lo = 0, hi = k;                       // first position with sel[pos] >= c
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (sel[mid] < c) lo = mid + 1; else hi = mid;
    }
    slotmap[c] = (lo < k && sel[lo] == c) ? lo : -1;
}

template <int MODE, int NT, int U, int WPE>
gf_status launch_shape(const gf_plan *pl, const FuseArgs &a, hipStream_t st)
{
    const int64_t blocks = static_cast<int64_t>(a.units) * pl->P;
    if (blocks <= 0) return GF_OK;
    const dim3 grid(static_cast<unsigned>(blocks)), block(NT);
    // fp16 gradients only matter to the modes that read gradients
    constexpr bool READS_G = MODE == MODE_ACCUM || MODE == MODE_FUSED || MODE == MODE_DENSE;
    const bool f16 = pl->wire == GF_WIRE_F16;
    if (READS_G && pl->grad == GF_WIRE_F16) {
        if constexpr (READS_G) {
            if (f16) hipLaunchKernelGGL((k_fuse<MODE, uint16_t, uint16_t, NT, U, WPE>), grid, block, 0, st, a);
            else hipLaunchKernelGGL((k_fuse<MODE, float, uint16_t, NT, U, WPE>), grid, block, 0, st, a);
        }
    } else if (f16) {
        hipLaunchKernelGGL((k_fuse<MODE, uint16_t, float, NT, U, WPE>), grid, block, 0, st, a);
    } else {
        hipLaunchKernelGGL((k_fuse<MODE, float, float, NT, U, WPE>), grid, block, 0, st, a);
    }
    GF_LAUNCH_CHECK();
    return GF_OK;
}

// Workgroup shape (measured on MI355X, P = 8..64 workers).  The in-place
// accumulate stream does best when a long tile is swept by 1024 threads that
// issue all 16 loads of a 32768-element stretch before the first store, and a
// short tile by small workgroups with 8 loads in flight per thread and two
// workgroups resident per SIMD set.  The dense cast (read fp32, write fp16
// elsewhere) prefers full occupancy.
template <int MODE>
gf_status launch(const gf_plan *pl, const FuseArgs &a, hipStream_t st)
{
#if defined(GF_FUSE_NT)
    return launch_shape<MODE, GF_FUSE_NT, GF_FUSE_U, GF_FUSE_WPE>(pl, a, st);
#else
    if constexpr (MODE == MODE_DENSE) return launch_shape<MODE, 512, 4, 0>(pl, a, st);
    if (pl->tile > 16384) return launch_shape<MODE, 1024, 8, 0>(pl, a, st);
    return launch_shape<MODE, 256, 8, 2>(pl, a, st);
#endif
}

}  // namespace

extern "C" gf_status gf_fuse_pack(const gf_plan *pl, uint32_t phase,
                                  const void *const *grads, const float *const *pools,
                                  float *const *residual,
                                  const int32_t *sel_idx, int32_t k,
                                  float loss_scale, float mu,
                                  void *const *sendbuf, float *chunk_l1,
                                  void *workspace, gf_stream stream)
{
    if (!pl) return GF_EINVAL;
    if (phase == 0 || (phase & ~(GF_PHASE_ACCUM | GF_PHASE_PACK))) return GF_EINVAL;
    const bool accum = phase & GF_PHASE_ACCUM, pack = phase & GF_PHASE_PACK;
    if (accum && ((grads != nullptr) == (pools != nullptr))) return GF_EINVAL;
    if (pack && !sendbuf) return GF_EINVAL;
    if (!residual && (!(accum && pack) || sel_idx || chunk_l1)) return GF_EINVAL;
    if ((sel_idx || chunk_l1) && pl->chunk == 0) return GF_EINVAL;
    if (chunk_l1 && !accum) return GF_EINVAL;
    if (sel_idx && pack && (k < 1 || k > pl->n_chunks)) return GF_EINVAL;
    const bool need_map = sel_idx && pack && (accum || mu != 1.0f);
    if (need_map && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))) return GF_EINVAL;
    if (!pl->on_device) return GF_ESTATE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    FuseArgs a{};
    a.tab = grads ? grads : reinterpret_cast<const void *const *>(pools);
    a.tab_stride = grads ? pl->m : 1;
    a.use_pieces = grads ? 1 : 0;
    a.residual = residual;
    a.sendbuf = sendbuf;
    a.chunk_l1 = chunk_l1;
    a.piece_start = pl->d_piece_start;
    a.pieces = pl->d_pieces;
    a.N = pl->N;
    a.tile = pl->tile;
    a.n_tiles = pl->n_tiles;
    a.units = pl->n_tiles;
    a.S = loss_scale;
    a.mu = mu;

    int32_t *slotmap = nullptr;
    if (need_map) {
        slotmap = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + gf_ws_slotmap_off());
        hipLaunchKernelGGL(k_slotmap, dim3((pl->n_chunks + GF_BLOCK - 1) / GF_BLOCK), dim3(GF_BLOCK), 0, st,
                           sel_idx, k, pl->n_chunks, slotmap);
        GF_LAUNCH_CHECK();
    }

    if (accum && !pack) {
        a.mu = 1.0f;                         // hg <- acc
        return launch<MODE_ACCUM>(pl, a, st);
    }
    if (accum && pack) {
        if (!residual) return launch<MODE_DENSE>(pl, a, st);
        a.slotmap = slotmap;                 // null: every chunk is sent, rank = chunk index
        return launch<MODE_FUSED>(pl, a, st);
    }
    // pack only: visit the selected chunks; the rest only if mu scales them
    a.sel_idx = sel_idx;
    a.units = sel_idx ? k : pl->n_tiles;
    gf_status rc = launch<MODE_PACK>(pl, a, st);
    if (rc != GF_OK || !sel_idx || mu == 1.0f) return rc;
    a.units = pl->n_tiles;
    a.slotmap = slotmap;
    return launch<MODE_SCALE>(pl, a, st);
}
