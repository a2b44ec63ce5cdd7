// gf_unpack_apply: reduced wire values back to fp32 times alpha, written into
// the gradient pool and/or scattered to the per-tensor buffers, only at the
// chunks that were sent (Section 2.5 second conversion; Section 3.2), plus the
// L1 norm of each written chunk for the next selection.
#include "gf_device.h"

namespace {

struct UnpackArgs {
    const void *reduced;
    const int32_t *sel_idx;        // NULL: tile index = block index
    float *out_pool;
    void *const *out_tensors;
    float *reduced_l1;
    const int32_t *piece_start;
    const gf_piece *pieces;
    int64_t N;
    int32_t tile;
    float alpha;
};

template <typename W>
__device__ __forceinline__ void run(const W *src_, float *dst_, int len, float alpha, double &l1)
{
    const GF_GLOBAL W *__restrict__ src = gf_global(src_);
    GF_GLOBAL float *__restrict__ dst = gf_global(dst_);
    using W4 = typename gf_wire4<W>::type;
    const bool vec = gf_aligned(src, sizeof(W4)) && gf_aligned(dst, 16);
    const int nvec = vec ? (len >> 2) : 0;
    const GF_GLOBAL W4 *s4 = reinterpret_cast<const GF_GLOBAL W4 *>(src);
    GF_GLOBAL gf_f32x4 *d4 = reinterpret_cast<GF_GLOBAL gf_f32x4 *>(dst);
    constexpr int U = 4;
    int v = threadIdx.x;
    for (; v + (U - 1) * GF_BLOCK < nvec; v += U * GF_BLOCK) {
        W4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = s4[v + u * GF_BLOCK];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float a, b, c, d;
            gf_unpack4(x[u], a, b, c, d);
            a *= alpha; b *= alpha; c *= alpha; d *= alpha;
            l1 += static_cast<double>(fabsf(a)); l1 += static_cast<double>(fabsf(b));
            l1 += static_cast<double>(fabsf(c)); l1 += static_cast<double>(fabsf(d));
            d4[v + u * GF_BLOCK] = gf_pack4(a, b, c, d);
        }
    }
    for (; v < nvec; v += GF_BLOCK) {
        float a, b, c, d;
        gf_unpack4(s4[v], a, b, c, d);
        a *= alpha; b *= alpha; c *= alpha; d *= alpha;
        l1 += static_cast<double>(fabsf(a)); l1 += static_cast<double>(fabsf(b));
        l1 += static_cast<double>(fabsf(c)); l1 += static_cast<double>(fabsf(d));
        d4[v] = gf_pack4(a, b, c, d);
    }
    for (int i = (nvec << 2) + threadIdx.x; i < len; i += GF_BLOCK) {
        const float a = gf_from_wire<W>(src[i]) * alpha;
        l1 += static_cast<double>(fabsf(a));
        dst[i] = a;
    }
}

template <typename W>
__global__ __launch_bounds__(GF_BLOCK) void k_unpack(const UnpackArgs a)
{
    const int j = blockIdx.x;
    const int tile = a.sel_idx ? a.sel_idx[j] : j;
    const int64_t tile_lo = static_cast<int64_t>(tile) * a.tile;
    const int64_t left = a.N - tile_lo;
    const int tile_len = left < a.tile ? static_cast<int>(left) : a.tile;
    const W *src = static_cast<const W *>(a.reduced) + static_cast<int64_t>(j) * a.tile;
    double l1 = 0.0, unused = 0.0;
    if (a.out_pool) run<W>(src, a.out_pool + tile_lo, tile_len, a.alpha, l1);
    if (a.out_tensors) {
        double &acc = a.out_pool ? unused : l1;     // count each element once
        const int pe = a.piece_start[tile + 1];
        for (int i = a.piece_start[tile]; i < pe; ++i) {
            const gf_piece pc = a.pieces[i];
            float *dst = static_cast<float *>(a.out_tensors[pc.tensor]) + pc.src_off;
            run<W>(src + pc.dst_rel, dst, pc.len, a.alpha, acc);
        }
    }
    const double s = gf_block_sum<GF_BLOCK>(l1);
    if (a.reduced_l1 && threadIdx.x == 0) a.reduced_l1[j] = static_cast<float>(s);
}

}  // namespace

extern "C" gf_status gf_unpack_apply(const gf_plan *pl, const void *reduced, int64_t L,
                                     const int32_t *sel_idx, int32_t k, float alpha,
                                     float *out_pool, void *const *out_tensors,
                                     float *reduced_l1, void *workspace, gf_stream stream)
{
    (void)workspace;
    if (!pl || !reduced || (!out_pool && !out_tensors)) return GF_EINVAL;
    int32_t blocks;
    if (sel_idx) {
        if (pl->chunk == 0 || k < 1 || k > pl->n_chunks) return GF_EINVAL;
        const int64_t C = pl->chunk;
        if (L <= (k - 1) * C || L > k * C) return GF_EINVAL;
        blocks = k;
    } else {
        if (L != pl->N || reduced_l1) return GF_EINVAL;
        blocks = pl->n_tiles;
    }
    if (!pl->on_device) return GF_ESTATE;

    UnpackArgs a{};
    a.reduced = reduced;
    a.sel_idx = sel_idx;
    a.out_pool = out_pool;
    a.out_tensors = out_tensors;
    a.reduced_l1 = reduced_l1;
    a.piece_start = pl->d_piece_start;
    a.pieces = pl->d_pieces;
    a.N = pl->N;
    a.tile = pl->tile;
    a.alpha = alpha;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (pl->wire == GF_WIRE_F16)
        hipLaunchKernelGGL((k_unpack<uint16_t>), dim3(blocks), dim3(GF_BLOCK), 0, st, a);
    else
        hipLaunchKernelGGL((k_unpack<float>), dim3(blocks), dim3(GF_BLOCK), 0, st, a);
    GF_LAUNCH_CHECK();
    return GF_OK;
}
