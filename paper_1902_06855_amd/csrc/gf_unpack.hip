// gf_unpack_apply / gf_unpack_sgd_update: reduced wire values back to fp32
// times alpha, only at the chunks that were sent (Section 2.5 second
// conversion; Section 3.2), written into the gradient pool and/or scattered to
// per-tensor buffers, plus the L1 norm of each written chunk for the next
// selection.  The update variant also applies the SGD-update half of
// Algorithm 1 (momentum SGD correction) in the same pass: at important chunks
// hu = momentum * hu + learning_rate * g and w = w + hu; everything else is
// left untouched (hu_t = hu_{t-1}, no weight update).
#include "gf_device.h"

namespace {

struct UnpackArgs {
    const void *reduced;
    const int32_t *sel_idx;        // NULL: tile index = block index
    float *out_pool;
    void *const *out_tensors;
    float *w_pool, *hu_pool;       // update variant, pool form
    void *const *w_tensors, *const *hu_tensors;   // update variant, per-tensor form
    uint16_t *wh_pool;             // update variant: FP16 copy of the weights (optional), pool form
    void *const *wh_tensors;       //                 the same, per-tensor form
    float *reduced_l1;
    const int32_t *piece_start;
    const gf_piece *pieces;
    int64_t N;
    int32_t tile;
    float alpha, momentum, lr;
    // optional filter (CSC plans): only the chunks of packed buckets whose last chunk lies in
    // [chunk_lo, chunk_hi); chunks_per_bucket = 0 switches it off
    int32_t k, chunks_per_bucket, chunk_lo, chunk_hi;
};

// log2 of the consecutive tiles one XCD takes
constexpr int UNPACK_GRP_SHIFT = 4;

// One contiguous run.  dst may be null in the update variant (gradient not kept); wh (the FP16
// copy of the weights, Section 2.5) may be null.
template <typename W, bool UPD, int NT>
__device__ __forceinline__ void run(const W *src_, float *dst_, float *hu_, float *w_, uint16_t *wh_, int len,
                                    const UnpackArgs &a, double &l1)
{
    const GF_GLOBAL W *__restrict__ src = gf_global(src_);
    GF_GLOBAL float *__restrict__ dst = gf_global(dst_);
    GF_GLOBAL float *__restrict__ hu = gf_global(hu_);
    GF_GLOBAL float *__restrict__ w = gf_global(w_);
    GF_GLOBAL uint16_t *__restrict__ wh = gf_global(wh_);
    using W4 = typename gf_wire4<W>::type;
    const float alpha = a.alpha, mom = a.momentum, lr = a.lr;
    bool vec = gf_aligned(src, sizeof(W4)) && (!dst || gf_aligned(dst, 16));
    if constexpr (UPD) vec = vec && gf_aligned(hu, 16) && gf_aligned(w, 16) && (!wh || gf_aligned(wh, 8));
    const int nvec = vec ? (len >> 2) : 0;
    // Streams go through buffer descriptors made for exactly this run: the reduced values were
    // just written by the ring kernel (cached loads); everything written here is not read again
    // in this iteration (streaming stores), as are the one-touch loads of hu and w.
    constexpr int WB = static_cast<int>(sizeof(W4));
    const uint32_t n4 = static_cast<uint32_t>(len) * 4u;
    const __amdgpu_buffer_rsrc_t sb = gf_make_buf(src, static_cast<uint32_t>(len) * sizeof(W));
    const __amdgpu_buffer_rsrc_t db = gf_make_buf(dst, dst ? n4 : 0u);
    const __amdgpu_buffer_rsrc_t hb = gf_make_buf(hu, UPD ? n4 : 0u);
    const __amdgpu_buffer_rsrc_t wb = gf_make_buf(w, UPD ? n4 : 0u);
    const __amdgpu_buffer_rsrc_t whb = gf_make_buf(wh, (UPD && wh) ? n4 / 2u : 0u);
    auto ld_src = [&](int v) {
        if constexpr (sizeof(W) == 2) return gf_buf_ld64u<GF_AUX_CACHED>(sb, v * WB);
        else return gf_buf_ld128<GF_AUX_CACHED>(sb, v * WB);
    };

    auto one = [&](int v, W4 x, gf_f32x4 hh, gf_f32x4 ww) {
        float g0, g1, g2, g3;
        gf_unpack4(x, g0, g1, g2, g3);
        g0 *= alpha; g1 *= alpha; g2 *= alpha; g3 *= alpha;
        l1 += static_cast<double>(fabsf(g0)); l1 += static_cast<double>(fabsf(g1));
        l1 += static_cast<double>(fabsf(g2)); l1 += static_cast<double>(fabsf(g3));
        if (dst) gf_buf_st<GF_AUX_STREAM>(gf_pack4(g0, g1, g2, g3), db, v * 16);
        if constexpr (UPD) {
            // every product and sum rounds on its own (no contraction)
            const gf_f32x4 hn = gf_pack4(mom * hh.x + lr * g0, mom * hh.y + lr * g1,
                                         mom * hh.z + lr * g2, mom * hh.w + lr * g3);
            gf_buf_st<GF_AUX_STREAM>(hn, hb, v * 16);
            const gf_f32x4 wn = gf_pack4(ww.x + hn.x, ww.y + hn.y, ww.z + hn.z, ww.w + hn.w);
            gf_buf_st<GF_AUX_STREAM>(wn, wb, v * 16);
            if (wh) gf_buf_st<GF_AUX_STREAM>(gf_pack4(gf_f32_to_h(wn.x), gf_f32_to_h(wn.y), gf_f32_to_h(wn.z),
                                                      gf_f32_to_h(wn.w)), whb, v * 8);
        }
    };

    constexpr int U = UPD ? 4 : 8;
    int v = threadIdx.x;
    for (; v + (U - 1) * NT < nvec; v += U * NT) {
        W4 x[U];
        gf_f32x4 hh[U] = {}, ww[U] = {};
#pragma unroll
        for (int u = 0; u < U; ++u) {
            x[u] = ld_src(v + u * NT);
            if constexpr (UPD) {
                hh[u] = gf_buf_ld128<GF_AUX_STREAM>(hb, (v + u * NT) * 16);
                ww[u] = gf_buf_ld128<GF_AUX_STREAM>(wb, (v + u * NT) * 16);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) one(v + u * NT, x[u], hh[u], ww[u]);
    }
    if (v < nvec) {
        // less than a full batch left: the same batch with the lanes past the end switched off
        W4 x[U] = {};
        gf_f32x4 hh[U] = {}, ww[U] = {};
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (v + u * NT < nvec) {
                x[u] = ld_src(v + u * NT);
                if constexpr (UPD) {
                    hh[u] = gf_buf_ld128<GF_AUX_STREAM>(hb, (v + u * NT) * 16);
                    ww[u] = gf_buf_ld128<GF_AUX_STREAM>(wb, (v + u * NT) * 16);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (v + u * NT < nvec) one(v + u * NT, x[u], hh[u], ww[u]);
    }
    for (int i = (nvec << 2) + threadIdx.x; i < len; i += NT) {
        const float g = gf_from_wire<W>(src[i]) * alpha;
        l1 += static_cast<double>(fabsf(g));
        if (dst) dst[i] = g;
        if constexpr (UPD) {
            const float hn = mom * hu[i] + lr * g;
            hu[i] = hn;
            const float wn = w[i] + hn;
            w[i] = wn;
            if (wh) wh[i] = gf_f32_to_h(wn);
        }
    }
}

template <typename W, bool UPD, int NT>
__global__ __launch_bounds__(NT) void k_unpack(const UnpackArgs a)
{
    const int j = gf_xcd_order(blockIdx.x, gridDim.x, UNPACK_GRP_SHIFT);
    if (a.chunks_per_bucket) {                       // uniform across the workgroup
        const int64_t after = (static_cast<int64_t>(j / a.chunks_per_bucket) + 1) * a.chunks_per_bucket;
        const int32_t c = a.sel_idx[(after < a.k ? after : a.k) - 1];
        if (c < a.chunk_lo || c >= a.chunk_hi) return;
    }
    const int tile = a.sel_idx ? a.sel_idx[j] : j;
    const int64_t tile_lo = static_cast<int64_t>(tile) * a.tile;
    const int64_t left = a.N - tile_lo;
    const int tile_len = left < a.tile ? static_cast<int>(left) : a.tile;
    const W *src = static_cast<const W *>(a.reduced) + static_cast<int64_t>(j) * a.tile;
    double l1 = 0.0, unused = 0.0;
    const bool pooled = a.out_pool || (UPD && a.w_pool);
    if (pooled) {
        float *out = a.out_pool ? a.out_pool + tile_lo : nullptr;
        if (UPD && a.w_pool)
            run<W, UPD, NT>(src, out, a.hu_pool + tile_lo, a.w_pool + tile_lo,
                            a.wh_pool ? a.wh_pool + tile_lo : nullptr, tile_len, a, l1);
        else run<W, false, NT>(src, out, nullptr, nullptr, nullptr, tile_len, a, l1);
    }
    if (a.out_tensors || (UPD && a.w_tensors)) {
        // per-tensor destinations: walk the pieces of this tile
        double &acc = pooled ? unused : l1;         // count each element once
        const int pe = a.piece_start[tile + 1];
        for (int i = a.piece_start[tile]; i < pe; ++i) {
            const gf_piece pc = a.pieces[i];
            float *dst = a.out_tensors ? static_cast<float *>(a.out_tensors[pc.tensor]) + pc.src_off : nullptr;
            if constexpr (UPD) {
                if (a.w_tensors) {
                    uint16_t *wh = a.wh_tensors ? static_cast<uint16_t *>(a.wh_tensors[pc.tensor]) + pc.src_off : nullptr;
                    run<W, true, NT>(src + pc.dst_rel, dst, static_cast<float *>(a.hu_tensors[pc.tensor]) + pc.src_off,
                                     static_cast<float *>(a.w_tensors[pc.tensor]) + pc.src_off, wh, pc.len, a, acc);
                    continue;
                }
            }
            if (dst) run<W, false, NT>(src + pc.dst_rel, dst, nullptr, nullptr, nullptr, pc.len, a, acc);
        }
    }
    const double s = gf_block_sum<NT>(l1);
    if (a.reduced_l1 && threadIdx.x == 0) a.reduced_l1[j] = static_cast<float>(s);
}

template <int NT>
gf_status launch_unpack(const gf_plan *pl, const UnpackArgs &a, int32_t blocks, bool update, hipStream_t st)
{
    const bool h = pl->wire == GF_WIRE_F16;
    if (update) {
        if (h) hipLaunchKernelGGL((k_unpack<uint16_t, true, NT>), dim3(blocks), dim3(NT), 0, st, a);
        else hipLaunchKernelGGL((k_unpack<float, true, NT>), dim3(blocks), dim3(NT), 0, st, a);
    } else {
        if (h) hipLaunchKernelGGL((k_unpack<uint16_t, false, NT>), dim3(blocks), dim3(NT), 0, st, a);
        else hipLaunchKernelGGL((k_unpack<float, false, NT>), dim3(blocks), dim3(NT), 0, st, a);
    }
    GF_LAUNCH_CHECK();
    return GF_OK;
}

gf_status unpack_common(const gf_plan *pl, UnpackArgs &a, int64_t L, int32_t k, bool update, gf_stream stream)
{
    int32_t blocks;
    if (a.sel_idx) {
        if (pl->chunk == 0 || k < 1 || k > pl->n_chunks) return GF_EINVAL;
        const int64_t C = pl->chunk;
        if (L <= (k - 1) * C || L > k * C) return GF_EINVAL;
        blocks = k;
    } else {
        if (L != pl->N || a.reduced_l1) return GF_EINVAL;
        blocks = pl->n_tiles;
    }
    if (!pl->on_device) return GF_ESTATE;
    GF_CHECK_DEVICE(pl);
    a.piece_start = pl->d_piece_start;
    a.pieces = pl->d_pieces;
    a.N = pl->N;
    a.tile = pl->tile;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // few, long tiles (the selected chunks of a CSC plan) get 1024 threads each so that a
    // couple of hundred workgroups still fill the chip
    if (pl->tile >= 16384) return launch_unpack<1024>(pl, a, blocks, update, st);
    return launch_unpack<GF_BLOCK>(pl, a, blocks, update, st);
}

}  // namespace

extern "C" gf_status gf_unpack_apply(const gf_plan *pl, const void *reduced, int64_t L,
                                     const int32_t *sel_idx, int32_t k, float alpha,
                                     float *out_pool, void *const *out_tensors,
                                     float *reduced_l1, void *workspace, gf_stream stream)
{
    (void)workspace;
    if (!pl || !reduced || (!out_pool && !out_tensors)) return GF_EINVAL;
    UnpackArgs a{};
    a.reduced = reduced;
    a.sel_idx = sel_idx;
    a.out_pool = out_pool;
    a.out_tensors = out_tensors;
    a.reduced_l1 = reduced_l1;
    a.alpha = alpha;
    return unpack_common(pl, a, L, k, false, stream);
}

extern "C" gf_status gf_unpack_range(const gf_plan *pl, const void *reduced, int64_t L,
                                     const int32_t *sel_idx, int32_t k, int32_t chunk_lo, int32_t chunk_hi,
                                     float alpha, float *out_pool, void *const *out_tensors,
                                     float *reduced_l1, void *workspace, gf_stream stream)
{
    (void)workspace;
    if (!pl || !reduced || !sel_idx || (!out_pool && !out_tensors)) return GF_EINVAL;
    if (pl->chunk == 0 || chunk_lo < 0 || chunk_hi > pl->n_chunks || chunk_lo > chunk_hi) return GF_EINVAL;
    if (chunk_lo == chunk_hi) return GF_OK;
    UnpackArgs a{};
    a.reduced = reduced;
    a.sel_idx = sel_idx;
    a.out_pool = out_pool;
    a.out_tensors = out_tensors;
    a.reduced_l1 = reduced_l1;
    a.alpha = alpha;
    a.k = k;
    a.chunks_per_bucket = static_cast<int32_t>(gf_csc_bucket_span(pl) / pl->chunk);
    a.chunk_lo = chunk_lo;
    a.chunk_hi = chunk_hi;
    return unpack_common(pl, a, L, k, false, stream);
}

extern "C" gf_status gf_unpack_sgd_update(const gf_plan *pl, const void *reduced, int64_t L,
                                          const int32_t *sel_idx, int32_t k, float alpha,
                                          float momentum, float learning_rate,
                                          float *w_pool, float *hu_pool,
                                          void *const *w_tensors, void *const *hu_tensors,
                                          void *w_half_pool, void *const *w_half_tensors,
                                          float *out_pool, float *reduced_l1,
                                          void *workspace, gf_stream stream)
{
    (void)workspace;
    if (!pl || !reduced) return GF_EINVAL;
    const bool pool_form = w_pool && hu_pool && !w_tensors && !hu_tensors;
    const bool tensor_form = w_tensors && hu_tensors && !w_pool && !hu_pool;
    if (pool_form == tensor_form) return GF_EINVAL;
    if ((pool_form && w_half_tensors) || (tensor_form && w_half_pool)) return GF_EINVAL;   // same form as w
    UnpackArgs a{};
    a.reduced = reduced;
    a.sel_idx = sel_idx;
    a.out_pool = out_pool;
    a.w_pool = w_pool; a.hu_pool = hu_pool;
    a.w_tensors = w_tensors; a.hu_tensors = hu_tensors;
    a.wh_pool = static_cast<uint16_t *>(w_half_pool); a.wh_tensors = w_half_tensors;
    a.reduced_l1 = reduced_l1;
    a.alpha = alpha; a.momentum = momentum; a.lr = learning_rate;
    return unpack_common(pl, a, L, k, true, stream);
}
