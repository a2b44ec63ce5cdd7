// gf_ring_reduce_sim: the elementwise arithmetic of ring allreduce
// (Section 2.4) over P send buffers resident in this GPU's memory.
//
// Reduce-scatter hop t moves segment (r - t) mod P from rank r to rank r + 1,
// which adds its own values and rounds to the wire type; segment s therefore
// ends as the left fold x_s + x_{s+1} + ... + x_{s-1}.  The kernel computes
// that fold directly: one thread owns 16 bytes of one segment, reads the same
// 16 bytes from all P buffers starting at worker s, and writes the result once
// (plus P copies when the all-gather outputs are requested).  A workgroup never
// crosses a segment border, so s and the P base pointers are wave-uniform.
//
// Hierarchical allreduce (Section 2.4) is the same kernel with another visiting
// order: the P ranks form M groups of G consecutive ranks, each group's values
// are folded along the chain that ends on its lowest rank (the master),
// y_g = x_{gG+1} + ... + x_{gG+G-1} + x_{gG}, and the M masters run the ring:
// there are M segments, and segment s ends as y_s + y_{s+1} + ... + y_{s-1}.
// G = 1 is the flat ring.
#include "gf_device.h"

namespace {

// log2 of the consecutive workgroups (8 KB of every send buffer each) one XCD takes
constexpr int RING_GRP_SHIFT = 5;

// A dense plan's send buffers (P * N wire elements) are far larger than the
// caches and are read exactly once: they are streamed.  The packed buffer of a
// CSC plan was written just before by gf_fuse_pack and is still cache-resident:
// ordinary loads.

struct RingArgs {
    const void *const *send;
    void *reduced;
    void *const *allgather;
    const gf_bucket_dev *buckets;     // dense plans
    const gf_ring_block *blocks;      // dense plans
    const int64_t *L_dev;
    int64_t L;
    int32_t P;
    int32_t M, G;                     // ring participants (= segments) and ranks per group; M * G = P
    int32_t blocks_per_segment;       // CSC plans: workgroups per segment of a full bucket
    int64_t bucket_span;              // CSC plans: elements per full bucket of the packed buffer
    // CSC plans, optional filter: only the buckets whose last chunk lies in [chunk_lo, chunk_hi)
    const int32_t *sel;               // the selection the buffer was packed with (ascending), or NULL: every bucket
    int32_t k, chunks_per_bucket, chunk_lo, chunk_hi;
};

template <typename W> struct vec16;
template <> struct vec16<uint16_t> { using type = gf_u32x4; static constexpr int n = 8; };
template <> struct vec16<float> { using type = gf_f32x4; static constexpr int n = 4; };

__device__ __forceinline__ gf_u32x4 hop16(gf_u32x4 a, gf_u32x4 b)
{
    gf_u32x4 r = {gf_hop_add_h2(a.x, b.x), gf_hop_add_h2(a.y, b.y),
                  gf_hop_add_h2(a.z, b.z), gf_hop_add_h2(a.w, b.w)};
    return r;
}
__device__ __forceinline__ gf_f32x4 hop16(gf_f32x4 a, gf_f32x4 b)
{
    gf_f32x4 r = {a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w};
    return r;
}

// Visiting order of the hierarchical fold: position pos = j * G + l stands for
// rank ((s + j) mod M) * G + ((l + 1) mod G).  `feed` takes the values in that
// order: the first of a group opens the group's partial sum, the last closes it
// into the ring's running sum.
struct HierWalk {
    int G, M, g, l, j;
    __device__ HierWalk(int s, int M_, int G_) : G(G_), M(M_), g(s), l(0), j(0) {}
    __device__ int rank() const { return g * G + (l + 1 == G ? 0 : l + 1); }
    __device__ void next()
    {
        if (++l == G) { l = 0; ++j; g = g + 1 == M ? 0 : g + 1; }
    }
};

template <typename T, typename Add>
__device__ __forceinline__ void hier_feed(T &v, T &y, const T &x, int l, int j, int G, Add add)
{
    y = l == 0 ? x : add(y, x);
    if (l + 1 == G) v = j == 0 ? y : add(v, y);
}

template <typename W, bool DENSE, bool HIER>
__global__ __launch_bounds__(GF_RING_GROUPS_PER_BLOCK) void k_ring(const RingArgs a)
{
    using V = typename vec16<W>::type;
    constexpr int A = vec16<W>::n;
    const int P = a.P;
    const int M = HIER ? a.M : P;     // segments per bucket
    int64_t lo, hi, seg;
    int s, bis;
    const uint32_t item = gf_xcd_order(blockIdx.x, gridDim.x, RING_GRP_SHIFT);
    if constexpr (DENSE) {
        const gf_ring_block rb = a.blocks[item];
        const gf_bucket_dev bk = a.buckets[rb.bucket];
        lo = bk.lo; hi = bk.hi; seg = bk.seg;
        s = rb.segment; bis = rb.block_in_segment;
    } else {
        // Packed buffer of a CSC plan.  All packed chunks have C elements (only the pool's
        // last chunk can be short, and it is packed last), so the lazy-allreduce rule "flush
        // when more than theta is waiting" closes a bucket every floor(theta / C) + 1 chunks:
        // buckets are [b * span, min(L, (b + 1) * span)).
        int64_t L = a.L;
        if (a.L_dev) { const int64_t d = *a.L_dev; L = d < 0 ? 0 : (d < L ? d : L); }
        const int per_bucket = M * a.blocks_per_segment;
        const int b = item / per_bucket;
        const int r = item - b * per_bucket;
        lo = static_cast<int64_t>(b) * a.bucket_span;
        if (lo >= L) return;
        if (a.sel) {
            // the bucket is complete once its last chunk has been packed: it is reduced by the
            // call whose range holds that chunk, and by no other
            const int64_t after = (static_cast<int64_t>(b) + 1) * a.chunks_per_bucket;
            const int32_t c = a.sel[(after < a.k ? after : a.k) - 1];
            if (c < a.chunk_lo || c >= a.chunk_hi) return;
        }
        hi = lo + a.bucket_span < L ? lo + a.bucket_span : L;
        const int64_t per = (hi - lo + M - 1) / M;
        seg = (per + A - 1) / A * A;
        s = r / a.blocks_per_segment;
        bis = r - s * a.blocks_per_segment;
    }
    const int64_t Lb = hi - lo;
    int64_t seg_lo = static_cast<int64_t>(s) * seg; if (seg_lo > Lb) seg_lo = Lb;
    int64_t seg_hi = seg_lo + seg; if (seg_hi > Lb) seg_hi = Lb;
    seg_lo += lo; seg_hi += lo;
    // 16-byte groups per workgroup = its thread count (fewer than the full 512 when a small
    // packed buffer would otherwise leave most of the chip idle)
    const int gpb = DENSE ? GF_RING_GROUPS_PER_BLOCK : static_cast<int>(blockDim.x);
    const int64_t e = seg_lo + (static_cast<int64_t>(bis) * gpb + threadIdx.x) * A;
    if (e >= seg_hi) return;
    const int n = seg_hi - e < A ? static_cast<int>(seg_hi - e) : A;

    // 128-bit path needs every buffer 16-byte aligned at this offset.  All
    // offsets of a segment differ from seg_lo by multiples of 16 bytes.
    unsigned mis = static_cast<unsigned>((seg_lo * sizeof(W)) & 15);
    for (int q = 0; q < P; ++q) mis |= static_cast<unsigned>(reinterpret_cast<uintptr_t>(a.send[q]) & 15);
    mis |= static_cast<unsigned>(reinterpret_cast<uintptr_t>(a.reduced) & 15);
    if (a.allgather)
        for (int q = 0; q < P; ++q) mis |= static_cast<unsigned>(reinterpret_cast<uintptr_t>(a.allgather[q]) & 15);

    if (mis == 0 && n == A) {
        // Buffer descriptors anchored at this workgroup's first element: the base is uniform,
        // each lane adds 16 bytes times its index, and nothing past the segment is reachable.
        constexpr int AUX = DENSE ? GF_AUX_STREAM : GF_AUX_CACHED;
        const int64_t blk = seg_lo + static_cast<int64_t>(bis) * gpb * A;
        const int64_t left = (seg_hi - blk) * static_cast<int64_t>(sizeof(W));
        const uint32_t bytes = left < gpb * 16 ? static_cast<uint32_t>(left) : static_cast<uint32_t>(gpb) * 16u;
        const int off = threadIdx.x * 16;
        auto ld = [&](int q) {
            const __amdgpu_buffer_rsrc_t r = gf_make_buf(gf_global(static_cast<const W *>(a.send[q])) + blk, bytes);
            return __builtin_bit_cast(V, gf_buf_ld128u<AUX>(r, off));
        };
        // Loads in flight per thread.  The big dense sweep runs best with one (measured at P = 8:
        // 6.6 TB/s against 6.4 with eight; plenty of wavefronts are resident and more requests in
        // flight only open more DRAM pages at once); the small packed buffer of a CSC plan is
        // latency-bound (a few dozen workgroups) and wants many.
        constexpr int U = DENSE ? 1 : 16;
        V v;
        if constexpr (HIER) {
            const int G = a.G;
            auto add = [](const V &p, const V &q) { return hop16(p, q); };
            HierWalk rd(s, M, G), ap(s, M, G);       // one walks ahead issuing loads, one applies them
            V y = {};
            v = y;
            // batches of up to U loads in flight; a short last batch keeps all of its loads in
            // flight too (the count is uniform across the workgroup)
            for (int pos = 0; pos < P; pos += U) {
                const int nb = P - pos < U ? P - pos : U;
                V x[U];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (u < nb) { x[u] = ld(rd.rank()); rd.next(); }
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (u < nb) { hier_feed(v, y, x[u], ap.l, ap.j, G, add); ap.next(); }
            }
        } else {
            int q = s;
            v = ld(q);
            for (int j = 1; j < P; j += U) {
                const int nb = P - j < U ? P - j : U;
                V x[U];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (u < nb) {
                        q = q + 1 == P ? 0 : q + 1;
                        x[u] = ld(q);
                    }
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (u < nb) v = hop16(v, x[u]);
            }
        }
        gf_buf_st<GF_AUX_CACHED>(__builtin_bit_cast(gf_u32x4, v),
                                 gf_make_buf(gf_global(static_cast<W *>(a.reduced)) + blk, bytes), off);
        if (a.allgather)
            for (int r = 0; r < P; ++r)
                gf_buf_st<GF_AUX_STREAM>(__builtin_bit_cast(gf_u32x4, v),
                                         gf_make_buf(gf_global(static_cast<W *>(a.allgather[r])) + blk, bytes), off);
    } else {
        for (int i = 0; i < n; ++i) {
            W v;
            if constexpr (HIER) {
                auto add = [](W p, W q) { return gf_hop_add(p, q); };
                HierWalk ap(s, M, a.G);
                W y = 0;
                v = 0;
                for (int pos = 0; pos < P; ++pos) {
                    hier_feed(v, y, static_cast<const W *>(a.send[ap.rank()])[e + i], ap.l, ap.j, a.G, add);
                    ap.next();
                }
            } else {
                int q = s;
                v = static_cast<const W *>(a.send[q])[e + i];
                for (int j = 1; j < P; ++j) {
                    q = q + 1 == P ? 0 : q + 1;
                    v = gf_hop_add(v, static_cast<const W *>(a.send[q])[e + i]);
                }
            }
            static_cast<W *>(a.reduced)[e + i] = v;
            if (a.allgather)
                for (int r = 0; r < P; ++r) static_cast<W *>(a.allgather[r])[e + i] = v;
        }
    }
}

}  // namespace

namespace {

gf_status ring_reduce(const gf_plan *pl, const void *const *sendbuf, int64_t L, const int64_t *L_dev,
                      const int32_t *sel_idx, int32_t k, int32_t chunk_lo, int32_t chunk_hi,
                      void *reduced, void *const *allgather_out, gf_stream stream)
{
    if (!pl || !sendbuf || !reduced || L < 0) return GF_EINVAL;
    const bool dense = pl->chunk == 0;
    if (sel_idx) {
        if (dense || k < 1 || k > pl->n_chunks || chunk_lo < 0 || chunk_hi > pl->n_chunks || chunk_lo > chunk_hi)
            return GF_EINVAL;
        if (L != static_cast<int64_t>(k) * pl->chunk) return GF_EINVAL;     // the capacity of k packed chunks
        if (chunk_lo == chunk_hi) return GF_OK;
    }
    if (dense && (L != pl->N || L_dev)) return GF_EINVAL;
    if (!dense && L > static_cast<int64_t>(pl->n_chunks) * pl->chunk) return GF_EINVAL;
    if (!pl->on_device) return GF_ESTATE;
    GF_CHECK_DEVICE(pl);
    hipStream_t st = static_cast<hipStream_t>(stream);

    RingArgs a{};
    a.send = sendbuf;
    a.reduced = reduced;
    a.allgather = allgather_out;
    a.L = L;
    a.L_dev = L_dev;
    a.sel = sel_idx;
    a.k = k;
    a.chunk_lo = chunk_lo;
    a.chunk_hi = chunk_hi;
    a.P = pl->P;
    a.M = pl->ring_M;
    a.G = pl->P / pl->ring_M;
    const bool hier = a.G > 1;
    const bool f16 = pl->wire == GF_WIRE_F16;
    const dim3 block(GF_RING_GROUPS_PER_BLOCK);
    if (dense) {
        a.buckets = pl->d_buckets;
        a.blocks = pl->d_ring_blocks;
        const size_t nb = pl->ring_blocks.size();
        if (nb == 0) return GF_OK;
        const dim3 grid(static_cast<unsigned>(nb));
        if (f16 && !hier) hipLaunchKernelGGL((k_ring<uint16_t, true, false>), grid, block, 0, st, a);
        else if (f16) hipLaunchKernelGGL((k_ring<uint16_t, true, true>), grid, block, 0, st, a);
        else if (!hier) hipLaunchKernelGGL((k_ring<float, true, false>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((k_ring<float, true, true>), grid, block, 0, st, a);
    } else {
        if (L == 0) return GF_OK;
        const int64_t A = gf_wire_granule(pl->wire);
        const int64_t span = gf_csc_bucket_span(pl);
        const int64_t full = span < L ? span : L;                      // longest bucket (upper bound with L_dev)
        const int64_t n_buckets = (L + span - 1) / span;
        const int64_t seg = gf_ring_segment_len(full, pl->ring_M, pl->wire);
        const int64_t groups = seg / A;
        // a small packed buffer is cut into smaller workgroups (down to one wavefront) until a
        // thousand of them exist: with 64 workgroups of 512 threads each CU's own load bandwidth
        // bounds the kernel (measured at P = 64, 0.5 MB per worker)
        int64_t gpb = GF_RING_GROUPS_PER_BLOCK;
        while (gpb > 64 && (groups + gpb - 1) / gpb * pl->ring_M * n_buckets < 1024) gpb /= 2;
        const int64_t bps = (groups + gpb - 1) / gpb;
        if (bps * pl->ring_M * n_buckets > (int64_t{1} << 30)) return GF_EINVAL;
        const dim3 block(static_cast<unsigned>(gpb));
        a.blocks_per_segment = static_cast<int32_t>(bps);
        a.bucket_span = span;
        a.chunks_per_bucket = static_cast<int32_t>(span / pl->chunk);
        const dim3 grid(static_cast<unsigned>(bps * pl->ring_M * n_buckets));
        if (f16 && !hier) hipLaunchKernelGGL((k_ring<uint16_t, false, false>), grid, block, 0, st, a);
        else if (f16) hipLaunchKernelGGL((k_ring<uint16_t, false, true>), grid, block, 0, st, a);
        else if (!hier) hipLaunchKernelGGL((k_ring<float, false, false>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((k_ring<float, false, true>), grid, block, 0, st, a);
    }
    GF_LAUNCH_CHECK();
    return GF_OK;
}

}  // namespace

extern "C" gf_status gf_ring_reduce_sim(const gf_plan *pl, const void *const *sendbuf, int64_t L,
                                        const int64_t *L_dev, void *reduced, void *const *allgather_out,
                                        void *workspace, gf_stream stream)
{
    (void)workspace;
    return ring_reduce(pl, sendbuf, L, L_dev, nullptr, 0, 0, 0, reduced, allgather_out, stream);
}

extern "C" gf_status gf_ring_reduce_range(const gf_plan *pl, const void *const *sendbuf, int64_t L,
                                          const int64_t *L_dev, const int32_t *sel_idx, int32_t k,
                                          int32_t chunk_lo, int32_t chunk_hi, void *reduced,
                                          void *const *allgather_out, void *workspace, gf_stream stream)
{
    (void)workspace;
    if (!sel_idx) return GF_EINVAL;
    return ring_reduce(pl, sendbuf, L, L_dev, sel_idx, k, chunk_lo, chunk_hi, reduced, allgather_out, stream);
}
