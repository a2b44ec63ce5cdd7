// gf_csc_iteration: one steady-state iteration of coarse-grained sparse
// communication in the paper's schedule (Section 3.2, Algorithm 1) as one host
// call: the four compute calls back to back on one stream.  Host code only; the
// kernels are those of the single calls.
#include "gf_internal.h"

extern "C" gf_status gf_csc_iteration(const gf_plan *pl, uint32_t modifiers,
                                      const void *const *grads, const float *const *pools,
                                      float *const *residual,
                                      int32_t *sel_idx, int32_t k, int32_t k_next, int64_t *packed_len,
                                      float loss_scale, float mu, void *const *sendbuf,
                                      void *reduced, void *const *allgather_out,
                                      float alpha, float *out_pool, void *const *out_tensors,
                                      float *reduced_l1, float *scores, uint8_t *mask,
                                      void *workspace, gf_stream stream)
{
    // Everything any of the four calls would reject is rejected here, before the first launch.
    if (!pl || pl->chunk == 0) return GF_EINVAL;
    if (modifiers & ~GF_PHASE_SLOTS) return GF_EINVAL;
    if ((grads != nullptr) == (pools != nullptr)) return GF_EINVAL;
    if (!residual || !sel_idx || !packed_len || !sendbuf || !reduced || !reduced_l1) return GF_EINVAL;
    if (!out_pool && !out_tensors) return GF_EINVAL;
    if (k < 1 || k > pl->n_chunks || k_next < 1 || k_next > pl->n_chunks) return GF_EINVAL;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return GF_EINVAL;
    if (!pl->on_device) return GF_ESTATE;
    GF_CHECK_DEVICE(pl);

    const int64_t cap = static_cast<int64_t>(k) * pl->chunk;      // capacity of k packed chunks
    gf_status st = gf_fuse_pack(pl, GF_PHASE_ACCUM | GF_PHASE_PACK | GF_PHASE_DEFER_NORMS | modifiers, grads, pools,
                                residual, sel_idx, k, loss_scale, mu, sendbuf, nullptr, workspace, stream);
    if (st != GF_OK) return st;
    st = gf_ring_reduce_sim(pl, sendbuf, cap, packed_len, reduced, allgather_out, workspace, stream);
    if (st != GF_OK) return st;
    st = gf_unpack_apply(pl, reduced, cap, sel_idx, k, alpha, out_pool, out_tensors, reduced_l1, workspace, stream);
    if (st != GF_OK) return st;
    return gf_chunk_score_select(pl, nullptr, reduced_l1, sel_idx, k, k_next, scores, sel_idx, mask, packed_len,
                                 workspace, stream);
}
