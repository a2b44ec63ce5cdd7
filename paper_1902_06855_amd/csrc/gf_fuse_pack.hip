// gf_fuse_pack: lazy-allreduce fusion folded into the read (Section 3.1), the
// allreduce-preprocess step of Algorithm 1 (g + hg, then hg = 0 or
// momentum * g), per-chunk L1 norms (Section 3.2) and the fp32 -> wire cast
// with loss scaling (Section 2.5), as one HBM-streaming pass per worker tile.
//
// A tile is a chunk of a CSC plan or a fixed slice of the pool of a dense plan;
// tiles longer than GF_FUSE_SUB elements are cut into sub-tiles of that length.
// One workgroup handles one (worker, tile, sub-tile) triple.  Whether the tile
// is sent is uniform across the workgroup, so each case runs its own
// straight-line inner loop of 128-bit loads and stores with several loads in
// flight.  With scattered per-tensor gradients a tile may be made of pieces of
// several tensors; their addresses are put in a small LDS table so that the
// sub-tile is still swept as one run.
//
// Workgroups are dealt to the eight XCDs round-robin by the hardware, and each
// XCD has its own L2.  The work list is therefore permuted so that a run of
// consecutive sub-tiles (1 MB of one worker's pool) is handled by one XCD:
// consecutive 32 KB sub-tiles spread over all XCDs use only part of each L2's
// channels and stream measurably slower.
#include <mutex>
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
    const gf_unit_src *unit_src; // [n_tiles * subs]
    double *l1_part;             // [P * n_tiles * subs] partial norms when subs > 1
    int64_t N;
    int32_t tile, n_tiles, units; // units: tiles to visit per worker
    int32_t tile_first;           // first tile of the visited range (0 unless a chunk range was asked for)
    int32_t sub, subs;            // sub-tile length (elements) and sub-tiles per tile
    uint32_t total;               // workgroups = P * units * subs
    int32_t grp_shift;            // log2 of the consecutive work items one XCD takes
    float S, mu;
};

// issue the first batch of historical-gradient loads before the gradients' address is known
constexpr bool FUSE_PREFETCH = true;

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

// One run of `len` elements.  res / snd are already offset to its first element;
// unused pointers are null.  Gradients and the historical gradient are touched
// exactly once per iteration, so they go around the caches (nontemporal); the
// send buffer is read back by the ring kernel right away and stays cacheable.
//
// Where the gradients live is found by `resolve(src)`, which returns 1 (source
// known, 128-bit path allowed), 0 (source known, element-wise only) or -1 (not
// a single source: nothing is done and false is returned).  With scattered
// tensors that takes a chain of dependent table look-ups, so the first batch of
// historical-gradient loads, whose address is known at once, is issued before it.
template <int F, typename W, typename GT, int NT, int U, typename Resolve>
__device__ __forceinline__ bool run(Resolve &&resolve, float *res_, W *snd_, int len, float S, float mu, double &l1)
{
    using G4 = typename gf_wire4<GT>::type;                // four gradients as stored
    GF_GLOBAL float *__restrict__ res = gf_global(res_);
    GF_GLOBAL W *__restrict__ snd = gf_global(snd_);
    using W4 = typename gf_wire4<W>::type;
    constexpr bool WRITES_RES = (F & (F_KEEP | F_ZERO)) != 0;
    bool vec = true;
    if constexpr ((F & F_RES) || WRITES_RES) vec = vec && gf_aligned(res, 16);
    if constexpr (F & F_SEND) vec = vec && gf_aligned(snd, sizeof(W4));
    const uint32_t run_bytes = static_cast<uint32_t>(len) * 4u;
    const __amdgpu_buffer_rsrc_t rb = gf_make_buf(res, ((F & F_RES) || WRITES_RES) ? run_bytes : 0u);

    constexpr bool PREFETCH = FUSE_PREFETCH && (F & F_RES) && (F & F_G);
    gf_f32x4 pre[U] = {};
    bool have_pre = PREFETCH && vec && U * NT <= (len >> 2);     // uniform: a whole first batch exists
    if constexpr (PREFETCH) {
        if (have_pre) {
#pragma unroll
            for (int u = 0; u < U; ++u) pre[u] = gf_buf_ld128<GF_AUX_STREAM>(rb, (threadIdx.x + u * NT) * 16);
        }
    }

    GradSrc<GT> src{nullptr, nullptr, nullptr, 0};
    const int how = resolve(src);
    if (how < 0) return false;
    vec = vec && how > 0;
    const int nvec = vec ? (len >> 2) : 0;
    auto g4 = [&](int v) { return reinterpret_cast<const GF_GLOBAL G4 *>(gf_global(src.at(v << 2))); };
    auto widen = [](G4 x) { float a, b, c, d; gf_unpack4(x, a, b, c, d); return gf_pack4(a, b, c, d); };

    // 128-bit sweep.  A direct source goes through buffer descriptors (one per stream, made
    // for exactly this run); a run pieced together from several tensors reads its gradients
    // through per-lane global addresses instead.
    constexpr int WB = static_cast<int>(sizeof(W4));      // bytes of four wire elements
    constexpr int GB = static_cast<int>(sizeof(G4));      // bytes of four gradients
    const __amdgpu_buffer_rsrc_t gb = gf_make_buf(gf_global(src.base), (F & F_G) && src.n == 0
                                                  ? static_cast<uint32_t>(len) * sizeof(GT) : 0u);
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
            if (have_pre) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if constexpr (F & F_G) gg[u] = load_g(v + u * NT);
                    rr[u] = pre[u];
                }
                have_pre = false;
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if constexpr (F & F_G) gg[u] = load_g(v + u * NT);
                    if constexpr (F & F_RES) rr[u] = gf_buf_ld128<GF_AUX_STREAM>(rb, (v + u * NT) * 16);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                gf_f32x4 ro; W4 so;
                elem4<F, W>(gg[u], rr[u], ro, so, S, mu, l1);
                if constexpr (WRITES_RES) gf_buf_st<GF_AUX_STREAM>(ro, rb, (v + u * NT) * 16);
                if constexpr (F & F_SEND) gf_buf_st<GF_AUX_CACHED>(so, sb, (v + u * NT) * WB);
            }
        }
        if (v < nvec) {
            // what is left is less than a full batch: the same batch with the lanes past the end
            // switched off, so that a ragged run still has all its loads in flight at once
            gf_f32x4 gg[U], rr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                gg[u] = gf_f32x4{}; rr[u] = gf_f32x4{};
                if (v + u * NT < nvec) {
                    if constexpr (F & F_G) gg[u] = load_g(v + u * NT);
                    if constexpr (F & F_RES) rr[u] = gf_buf_ld128<GF_AUX_STREAM>(rb, (v + u * NT) * 16);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (v + u * NT < nvec) {
                    gf_f32x4 ro; W4 so;
                    elem4<F, W>(gg[u], rr[u], ro, so, S, mu, l1);
                    if constexpr (WRITES_RES) gf_buf_st<GF_AUX_STREAM>(ro, rb, (v + u * NT) * 16);
                    if constexpr (F & F_SEND) gf_buf_st<GF_AUX_CACHED>(so, sb, (v + u * NT) * WB);
                }
            }
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
    return true;
}

constexpr int MAX_FLAT_PIECES = 64;   // more pieces than this in one run are walked one by one

// What a workgroup needs from the tables, fetched in one go at its start (every
// address here depends on the kernel arguments and the work item only).
template <typename GT>
struct Fetched {
    float *res_p;            // residual[p]
    void *snd_p;             // sendbuf[p]
    const GT *pool_p;        // tab[p * tab_stride]: the worker's pool, or its first tensor
    gf_unit_src us;          // single-tensor source of this sub-tile, if any
};

// Elements [lo, lo + len) of tile `tile` of worker p (lo a multiple of 4, the range inside the tile).
template <int F, typename W, typename GT, int NT, int U>
__device__ __forceinline__ void tile_body(const FuseArgs &a, const Fetched<GT> &f, int p, int tile, int64_t slot,
                                          int lo, int len, double &l1)
{
    constexpr unsigned GALIGN = 4 * sizeof(GT);            // alignment the vector path needs
    if (len <= 0) return;                                  // sub-tile past the end of a short last tile
    const int64_t tile_lo = static_cast<int64_t>(tile) * a.tile;
    constexpr bool USES_RES = (F & (F_RES | F_KEEP | F_ZERO)) != 0;
    float *res = USES_RES ? f.res_p + tile_lo + lo : nullptr;
    W *snd = (F & F_SEND) ? static_cast<W *>(f.snd_p) + slot * a.tile + lo : nullptr;
    if constexpr ((F & F_G) == 0) {
        run<F, W, GT, NT, U>([](GradSrc<GT> &) { return 1; }, res, snd, len, a.S, a.mu, l1);
        return;
    }
    if (!a.use_pieces) {
        run<F, W, GT, NT, U>([&](GradSrc<GT> &src) {
            src.base = f.pool_p + tile_lo + lo;
            return gf_aligned(src.base, GALIGN) ? 1 : 0;
        }, res, snd, len, a.S, a.mu, l1);
        return;
    }
    const GT *const *tab = reinterpret_cast<const GT *const *>(a.tab) + static_cast<int64_t>(p) * a.tab_stride;
    if (f.us.tensor >= 0) {                                // the whole range lies inside one tensor
        run<F, W, GT, NT, U>([&](GradSrc<GT> &src) {
            src.base = tab[f.us.tensor] + f.us.src_off;
            return gf_aligned(src.base, GALIGN) ? 1 : 0;
        }, res, snd, len, a.S, a.mu, l1);
        return;
    }
    __shared__ const GT *s_ptr[MAX_FLAT_PIECES];
    __shared__ int s_end[MAX_FLAT_PIECES];
    int ps = 0, pe = 0;
    bool used_lds = false;
    const bool done = run<F, W, GT, NT, U>([&](GradSrc<GT> &src) {
        // pieces of the tile that reach into [lo, lo + len)
        ps = a.piece_start[tile]; pe = a.piece_start[tile + 1];
        if (a.subs > 1) {
            while (ps < pe && a.pieces[ps].dst_rel + a.pieces[ps].len <= lo) ++ps;
            while (pe > ps && a.pieces[pe - 1].dst_rel >= lo + len) --pe;
        }
        const int np = pe - ps;
        if (np > MAX_FLAT_PIECES) return -1;
        // Several tensors meet in this run: publish where each piece lives, then sweep
        // it as if it were one run.
        int misaligned = 0;
        if (static_cast<int>(threadIdx.x) < np) {
            const gf_piece pc = a.pieces[ps + threadIdx.x];
            const GT *q = tab[pc.tensor] + pc.src_off;
            s_ptr[threadIdx.x] = q - (pc.dst_rel - lo);          // element x of the range is s_ptr[i][x]
            s_end[threadIdx.x] = pc.dst_rel + pc.len - lo;
            misaligned = !gf_aligned(q, GALIGN) || (pc.dst_rel & 3);
        }
        const bool vec = !__syncthreads_or(misaligned);
        src.ptr = s_ptr; src.end = s_end; src.n = np;
        used_lds = true;
        return vec ? 1 : 0;
    }, res, snd, len, a.S, a.mu, l1);
    if (used_lds) __syncthreads();             // the table is reused by the next caller
    if (done) return;
    for (int i = ps; i < pe; ++i) {
        const gf_piece pc = a.pieces[i];
        const int b = pc.dst_rel > lo ? pc.dst_rel : lo;                       // clipped to the range
        const int e = pc.dst_rel + pc.len < lo + len ? pc.dst_rel + pc.len : lo + len;
        run<F, W, GT, NT, U>([&](GradSrc<GT> &src) {
            src.base = tab[pc.tensor] + pc.src_off + (b - pc.dst_rel);
            return gf_aligned(src.base, GALIGN) ? 1 : 0;
        }, USES_RES ? res + (b - lo) : nullptr, (F & F_SEND) ? snd + (b - lo) : nullptr, e - b, a.S, a.mu, l1);
    }
}

// One workgroup per (worker, tile, sub-tile).  WPE caps the wavefronts resident
// per SIMD (0 = no cap): fewer resident workgroups mean fewer DRAM pages open at
// once, which the in-place read-read-write stream rewards.
template <int MODE, typename W, typename GT, int NT, int U, int WPE>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WPE ? WPE : 1, WPE ? WPE : 8)))
void k_fuse(const FuseArgs a)
{
    const uint32_t item = gf_xcd_order(blockIdx.x, a.total, a.grp_shift);
    const uint32_t per_worker = static_cast<uint32_t>(a.units) * static_cast<uint32_t>(a.subs);
    const int p = item / per_worker;
    const uint32_t r = item - p * per_worker;
    const int u = a.subs == 1 ? r : r / a.subs;
    const int sub = a.subs == 1 ? 0 : r - u * a.subs;
    int tile = a.tile_first + u;
    int64_t slot = tile;
    if constexpr (MODE == MODE_PACK) {
        if (a.sel_idx) { tile = a.sel_idx[u]; slot = u; }
    }
    // One round of table look-ups, issued together.  Unused entries read a valid dummy
    // location instead of branching, so that none of them waits for another.
    Fetched<GT> f;
    constexpr bool HAS_RES = MODE != MODE_DENSE, HAS_SND = MODE == MODE_FUSED || MODE == MODE_DENSE || MODE == MODE_PACK;
    constexpr bool HAS_G = MODE == MODE_ACCUM || MODE == MODE_FUSED || MODE == MODE_DENSE;
    const int32_t *slot_at = a.piece_start;                  // always a readable int32
    if constexpr (MODE == MODE_FUSED || MODE == MODE_SCALE) {
        if (a.slotmap) slot_at = a.slotmap + tile;
    }
    const int32_t slot_read = *slot_at;
    f.res_p = HAS_RES ? a.residual[p] : nullptr;
    f.snd_p = HAS_SND ? a.sendbuf[p] : nullptr;
    f.pool_p = HAS_G ? static_cast<const GT *>(a.tab[static_cast<int64_t>(p) * a.tab_stride]) : nullptr;
    f.us = gf_unit_src{0, -1, 0};
    if constexpr (HAS_G) f.us = a.unit_src[static_cast<int64_t>(tile) * a.subs + sub];
    {
        // All of the above are scalar loads that return together.  Naming every result here, in
        // one place, keeps the compiler from waiting for the first of them (the slot, which
        // decides a branch) before it has issued the others.
        uint64_t r0 = reinterpret_cast<uint64_t>(f.res_p), s0 = reinterpret_cast<uint64_t>(f.snd_p);
        uint64_t p0 = reinterpret_cast<uint64_t>(f.pool_p), o0 = static_cast<uint64_t>(f.us.src_off);
        int32_t t0 = f.us.tensor, sl = slot_read;
        asm volatile("" : "+s"(r0), "+s"(s0), "+s"(p0), "+s"(o0), "+s"(t0), "+s"(sl));
        f.res_p = reinterpret_cast<float *>(r0); f.snd_p = reinterpret_cast<void *>(s0);
        f.pool_p = reinterpret_cast<const GT *>(p0); f.us.src_off = static_cast<int64_t>(o0); f.us.tensor = t0;
        if constexpr (MODE == MODE_FUSED || MODE == MODE_SCALE) {
            if (a.slotmap) slot = sl;
        }
    }
    const int64_t left = a.N - static_cast<int64_t>(tile) * a.tile;
    const int tile_len = left < a.tile ? static_cast<int>(left) : a.tile;
    const int lo = sub * a.sub;                               // may lie past a short last tile
    int len = tile_len - lo;
    len = len < 0 ? 0 : (len < a.sub ? len : a.sub);
    double l1 = 0.0;
    if constexpr (MODE == MODE_ACCUM) tile_body<F_G | F_RES | F_KEEP | F_L1, W, GT, NT, U>(a, f, p, tile, 0, lo, len, l1);   // mu = 1 here
    if constexpr (MODE == MODE_FUSED) {
        if (slot >= 0) tile_body<F_G | F_RES | F_SEND | F_ZERO | F_L1, W, GT, NT, U>(a, f, p, tile, slot, lo, len, l1);
        else tile_body<F_G | F_RES | F_KEEP | F_L1, W, GT, NT, U>(a, f, p, tile, 0, lo, len, l1);
    }
    if constexpr (MODE == MODE_DENSE) tile_body<F_G | F_SEND, W, GT, NT, U>(a, f, p, tile, slot, lo, len, l1);
    if constexpr (MODE == MODE_PACK) tile_body<F_RES | F_SEND | F_ZERO, W, GT, NT, U>(a, f, p, tile, slot, lo, len, l1);
    if constexpr (MODE == MODE_SCALE) {
        if (slot < 0) tile_body<F_RES | F_KEEP, W, GT, NT, U>(a, f, p, tile, 0, lo, len, l1);
    }
    if constexpr (MODE == MODE_ACCUM || MODE == MODE_FUSED) {
        const double s = gf_block_sum<NT>(l1);
        if (threadIdx.x == 0) {
            const int64_t c = static_cast<int64_t>(p) * a.n_tiles + tile;
            if (a.l1_part) a.l1_part[c * a.subs + sub] = s;          // finished later, in a fixed order
            else if (a.chunk_l1) a.chunk_l1[c] = static_cast<float>(s);
        }
    }
}

// chunk_l1[c] = sum of the chunk's sub-tile norms, first sub-tile first (fp64), rounded once,
// for chunks [first, first + count) of every worker.
__global__ __launch_bounds__(GF_BLOCK) void k_l1_combine(const double *__restrict__ part, int32_t P, int32_t n_tiles,
                                                         int32_t first, int32_t count, int32_t subs,
                                                         float *__restrict__ chunk_l1)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * GF_BLOCK + threadIdx.x;
    if (i >= static_cast<int64_t>(P) * count) return;
    const int64_t p = i / count;
    const int64_t c = p * n_tiles + first + (i - p * count);
    double s = part[c * subs];
    for (int j = 1; j < subs; ++j) s += part[c * subs + j];
    chunk_l1[c] = static_cast<float>(s);
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
gf_status launch_shape(const gf_plan *pl, FuseArgs a, int grp_shift, hipStream_t st)
{
    const int64_t blocks = static_cast<int64_t>(a.units) * a.subs * pl->P;
    if (blocks <= 0) return GF_OK;
    if (blocks > (int64_t{1} << 30)) return GF_EINVAL;
    a.total = static_cast<uint32_t>(blocks);
    a.grp_shift = grp_shift;
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

// Workgroup shape (measured on MI355X, P = 8..64 workers, scattered tensors and
// pools, with the XCD-ordered work list): 256 threads that issue all 16 loads of
// an 8192-element sub-tile before the first store, two workgroups resident per
// SIMD set, runs of 32 sub-tiles (1 MB of a worker's pool) per XCD.
constexpr int FUSE_GRP_SHIFT = 5, DENSE_GRP_SHIFT = 5;
template <int MODE>
gf_status launch(const gf_plan *pl, const FuseArgs &a, hipStream_t st)
{
    if constexpr (MODE == MODE_DENSE) return launch_shape<MODE, 256, 8, 2>(pl, a, DENSE_GRP_SHIFT, st);
    // Shorter chunks put fewer bytes in flight per workgroup (every workgroup still issues all its
    // loads before its first store), so more of them must be resident for the same bytes in
    // flight per CU: four per SIMD set for up to 4096 elements, no cap below that (measured on the
    // ResNet-50-shaped set at P = 16: 5.8 -> 6.2 TB/s at 4096, 4.1 -> 6.1 TB/s at 2048).
    if (a.sub <= 2048) return launch_shape<MODE, 256, 4, 0>(pl, a, FUSE_GRP_SHIFT, st);
    if (a.sub <= 4096) return launch_shape<MODE, 256, 4, 4>(pl, a, FUSE_GRP_SHIFT, st);
    return launch_shape<MODE, 256, 8, 2>(pl, a, FUSE_GRP_SHIFT, st);
}

}  // namespace

// Scratch of gf_fuse_pack_static: one copy per GPU, part of the code object, held until the
// process ends.  Host code never uses this name as an address; it asks the runtime where the
// array lives on the current device and passes that pointer to the kernels.
static __device__ __align__(256) unsigned char scratch[GF_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void *scratch_ptr[MAX_DEVICES];        // device address of `scratch` on each GPU, once looked up

// Address of this GPU's copy of `scratch` (looked up once per device, with that device current).
gf_status static_scratch(void **out)
{
    int dev = -1;
    GF_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return GF_EINVAL;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        GF_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return GF_EHIP;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return GF_OK;
}

// Chunks [chunk_lo, chunk_hi) of every worker (the whole pool for a dense plan).
gf_status fuse_pack(const gf_plan *pl, uint32_t phase, const void *const *grads, const float *const *pools,
                    float *const *residual, const int32_t *sel_idx, int32_t k, float loss_scale, float mu,
                    void *const *sendbuf, float *chunk_l1, int32_t chunk_lo, int32_t chunk_hi,
                    void *workspace, gf_stream stream)
{
    if (!pl) return GF_EINVAL;
    constexpr uint32_t KNOWN = GF_PHASE_ACCUM | GF_PHASE_PACK | GF_PHASE_SLOTS | GF_PHASE_DEFER_NORMS;
    if ((phase & (GF_PHASE_ACCUM | GF_PHASE_PACK)) == 0 || (phase & ~KNOWN)) return GF_EINVAL;
    const bool accum = phase & GF_PHASE_ACCUM, pack = phase & GF_PHASE_PACK;
    const bool slots_ready = phase & GF_PHASE_SLOTS, defer = phase & GF_PHASE_DEFER_NORMS;
    if (accum && ((grads != nullptr) == (pools != nullptr))) return GF_EINVAL;
    if (pack && !sendbuf) return GF_EINVAL;
    if (!residual && (!(accum && pack) || sel_idx || chunk_l1)) return GF_EINVAL;
    if ((sel_idx || chunk_l1 || defer) && pl->chunk == 0) return GF_EINVAL;
    if ((chunk_l1 || defer) && !accum) return GF_EINVAL;
    if (defer && !residual) return GF_EINVAL;
    if (sel_idx && pack && (k < 1 || k > pl->n_chunks)) return GF_EINVAL;
    if (slots_ready && !(sel_idx && pack)) return GF_EINVAL;
    if (chunk_lo < 0 || chunk_hi > pl->n_tiles || chunk_lo > chunk_hi) return GF_EINVAL;
    const bool whole = chunk_lo == 0 && chunk_hi == pl->n_tiles;
    if (!whole && (pl->chunk == 0 || !accum)) return GF_EINVAL;      // a range needs chunks and the gradient pass
    const bool need_map = sel_idx && pack && (accum || mu != 1.0f);
    const int32_t subs = gf_fuse_subs(pl);
    const bool need_part = defer || (chunk_l1 && subs > 1);
    if ((need_map || need_part) && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))) return GF_EINVAL;
    if (!pl->on_device) return GF_ESTATE;
    GF_CHECK_DEVICE(pl);

    hipStream_t st = static_cast<hipStream_t>(stream);
    FuseArgs a{};
    a.tab = grads ? grads : reinterpret_cast<const void *const *>(pools);
    a.tab_stride = grads ? pl->m : 1;
    a.use_pieces = grads ? 1 : 0;
    a.residual = residual;
    a.sendbuf = sendbuf;
    a.chunk_l1 = defer ? nullptr : chunk_l1;
    a.piece_start = pl->d_piece_start;
    a.pieces = pl->d_pieces;
    a.unit_src = pl->d_unit_src;
    a.N = pl->N;
    a.tile = pl->tile;
    a.n_tiles = pl->n_tiles;
    a.tile_first = chunk_lo;
    a.units = chunk_hi - chunk_lo;
    a.sub = gf_fuse_sub_len(pl);
    a.subs = subs;
    if (need_part) a.l1_part = reinterpret_cast<double *>(static_cast<char *>(workspace) + gf_ws_l1part_off(pl));
    a.S = loss_scale;
    a.mu = mu;
    if (a.units == 0) return GF_OK;
    auto combine = [&](gf_status rc) {
        if (rc != GF_OK || defer || !(chunk_l1 && subs > 1)) return rc;
        const int64_t n_norms = static_cast<int64_t>(pl->P) * a.units;
        hipLaunchKernelGGL(k_l1_combine, dim3(static_cast<unsigned>((n_norms + GF_BLOCK - 1) / GF_BLOCK)), dim3(GF_BLOCK),
                           0, st, a.l1_part, pl->P, pl->n_tiles, chunk_lo, a.units, subs, chunk_l1);
        GF_LAUNCH_CHECK();
        return GF_OK;
    };

    int32_t *slotmap = nullptr;
    if (need_map) {
        slotmap = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + gf_ws_slotmap_off());
        if (!slots_ready) {
            hipLaunchKernelGGL(k_slotmap, dim3((pl->n_chunks + GF_BLOCK - 1) / GF_BLOCK), dim3(GF_BLOCK), 0, st,
                               sel_idx, k, pl->n_chunks, slotmap);
            GF_LAUNCH_CHECK();
        }
    }

    if (accum && !pack) {
        a.mu = 1.0f;                         // hg <- acc
        return combine(launch<MODE_ACCUM>(pl, a, st));
    }
    if (accum && pack) {
        if (!residual) return launch<MODE_DENSE>(pl, a, st);
        a.slotmap = slotmap;                 // null: every chunk is sent, rank = chunk index
        return combine(launch<MODE_FUSED>(pl, a, st));
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
    return fuse_pack(pl, phase, grads, pools, residual, sel_idx, k, loss_scale, mu, sendbuf, chunk_l1,
                     0, pl->n_tiles, workspace, stream);
}

extern "C" gf_status gf_fuse_pack_range(const gf_plan *pl, uint32_t phase,
                                        const void *const *grads, const float *const *pools,
                                        float *const *residual,
                                        const int32_t *sel_idx, int32_t k,
                                        float loss_scale, float mu,
                                        void *const *sendbuf, float *chunk_l1,
                                        int32_t chunk_lo, int32_t chunk_hi,
                                        void *workspace, gf_stream stream)
{
    if (!pl || pl->chunk == 0) return GF_EINVAL;
    return fuse_pack(pl, phase, grads, pools, residual, sel_idx, k, loss_scale, mu, sendbuf, chunk_l1,
                     chunk_lo, chunk_hi, workspace, stream);
}

extern "C" gf_status gf_fuse_pack_static(const gf_plan *pl, uint32_t phase,
                                         const void *const *grads, const float *const *pools,
                                         float *const *residual,
                                         const int32_t *sel_idx, int32_t k,
                                         float loss_scale, float mu,
                                         void *const *sendbuf, float *chunk_l1, gf_stream stream)
{
    if (!pl) return GF_EINVAL;
    // the scratch is private to this entry point: nothing another call left in a workspace is in it
    if (phase & (GF_PHASE_SLOTS | GF_PHASE_DEFER_NORMS)) return GF_EINVAL;
    if (gf_ws_total_bytes(pl) > static_cast<size_t>(GF_STATIC_SCRATCH_BYTES)) return GF_ELIMIT;
    void *ws = nullptr;
    const gf_status rc = static_scratch(&ws);
    if (rc != GF_OK) return rc;
    return fuse_pack(pl, phase, grads, pools, residual, sel_idx, k, loss_scale, mu, sendbuf, chunk_l1,
                     0, pl->n_tiles, ws, stream);
}
