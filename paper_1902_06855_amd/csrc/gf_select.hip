// gf_chunk_score_select: importance scores and the important-chunk set of
// Section 3.2.  The paper exchanges the per-chunk norms with a small allreduce;
// with all P norm rows in one memory that is a column sum.  The k largest
// scores are then found by a most-significant-byte-first radix select in LDS
// (no sort, no host round trip) and emitted in ascending chunk order by an
// ordered compaction; equal scores go to the lower chunk index.
#include "gf_device.h"

namespace {

constexpr int SEL_T = 1024;   // threads of the single selecting workgroup

// score[c]: chunks that went through this iteration's allreduce (c = prev_sel[j]) are scored by
// the norm of the (identical) reduced values, each GPU dividing it by the GPU count before the
// norms are summed over GPUs; every other chunk by the sum of the workers' local norms, rows
// added in ascending order.
// The local norms come either finished (l1, one float per worker and chunk) or, when gf_fuse_pack
// left them in the workspace, as per-sub-tile partial sums (part, `subs` doubles per worker and
// chunk) that are finished here exactly as gf_fuse_pack would have: sub-tiles added in ascending
// order in fp64, rounded once to fp32.
// SUBS: -1 finished norms; 1..4 that many partial sums per norm; 0 any number of them (`subs`).
__device__ __forceinline__ float sent_score(float reduced_norm, int32_t P)
{
    const double share = static_cast<double>(reduced_norm) / static_cast<double>(P);
    double s = 0.0;
    for (int p = 0; p < P; ++p) s += share;
    return static_cast<float>(s);
}

template <int SUBS>
__device__ __forceinline__ float local_score(const float *__restrict__ l1, const double *__restrict__ part,
                                             int32_t subs, int32_t P, int32_t nc, int c)
{
    // the norm of worker p, finished
    auto norm = [&](int p) {
        if constexpr (SUBS < 0) {
            return l1[static_cast<int64_t>(p) * nc + c];
        } else {
            const int n_sub = SUBS > 0 ? SUBS : subs;
            const double *q = part + (static_cast<int64_t>(p) * nc + c) * n_sub;
            double n = q[0];
            if constexpr (SUBS > 0) {
#pragma unroll
                for (int i = 1; i < SUBS; ++i) n += q[i];
            } else {
                for (int i = 1; i < n_sub; ++i) n += q[i];
            }
            return static_cast<float>(n);
        }
    };
    // several workers' loads are in flight at a time; the additions keep the order of the workers
    constexpr int B = SUBS <= 1 ? 16 : 8;
    double s = 0.0;
    int p = 0;
    for (; p + B <= P; p += B) {
        float x[B];
#pragma unroll
        for (int u = 0; u < B; ++u) x[u] = norm(p + u);
#pragma unroll
        for (int u = 0; u < B; ++u) s += static_cast<double>(x[u]);
    }
    for (; p < P; ++p) s += static_cast<double>(norm(p));
    return static_cast<float>(s);
}

template <int SUBS>
__global__ __launch_bounds__(GF_BLOCK) void k_score(const float *__restrict__ l1, const double *__restrict__ part,
                                                    int32_t subs, int32_t P, int32_t nc,
                                                    const float *__restrict__ red_l1,
                                                    const int32_t *__restrict__ prev_sel, int32_t k_prev,
                                                    float *__restrict__ score)
{
    const int c = blockIdx.x * GF_BLOCK + threadIdx.x;
    if (c >= nc) return;
    if (prev_sel) {
        int lo = 0, hi = k_prev;                  // first position with prev_sel[pos] >= c (ascending list)
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (prev_sel[mid] < c) lo = mid + 1; else hi = mid;
        }
        if (lo < k_prev && prev_sel[lo] == c) {
            score[c] = sent_score(red_l1[lo], P);
            return;
        }
    }
    score[c] = local_score<SUBS>(l1, part, subs, P, nc, c);
}

// Monotone map from float order to unsigned order.  A score that is not a number (of either
// sign, any payload) gets the largest key: such chunks rank above every number and tie.
__device__ __forceinline__ uint32_t ord_key(float f)
{
    uint32_t b = __float_as_uint(f);
    if ((b & 0x7fffffffu) > 0x7f800000u) return 0xffffffffu;
    if (b == 0x80000000u) b = 0;                             // -0 compares equal to +0
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(v, o, 64);
        if (lane >= o) v += t;
    }
    return v;
}

// Exclusive scan over the SEL_T threads; *total receives the sum (all threads).
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *wave_tot, uint32_t *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t incl = wave_incl_scan(v);
    __syncthreads();                               // wave_tot may still be read from a previous call
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < SEL_T / 64; ++w) {
        const uint32_t t = wave_tot[w];
        if (w < wave) before += t;
        all += t;
    }
    *total = all;
    return before + incl - v;
}

__global__ __launch_bounds__(SEL_T) void k_select(const float *__restrict__ score, int32_t nc, int32_t k,
                                                  int32_t C, int64_t N,
                                                  int32_t *__restrict__ sel, uint8_t *__restrict__ mask,
                                                  int64_t *__restrict__ packed_len, int32_t *__restrict__ slotmap)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wave_tot[SEL_T / 64];
    __shared__ uint32_t s_bin, s_remaining;
    const int tid = threadIdx.x;

    // ---- key of the k-th largest score, one byte per pass
    uint32_t prefix = 0, decided = 0, remaining = static_cast<uint32_t>(k);
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int c = tid; c < nc; c += SEL_T) {
            const uint32_t key = ord_key(score[c]);
            if ((key & decided) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        // thread t looks at bin 255 - t: a prefix sum over t is a count of keys in higher bins
        const uint32_t mine = tid < 256 ? hist[255 - tid] : 0u;
        uint32_t total;
        const uint32_t above = block_excl_scan(mine, wave_tot, &total);
        if (tid < 256 && above < remaining && above + mine >= remaining) {
            s_bin = static_cast<uint32_t>(255 - tid);
            s_remaining = remaining - above;
        }
        __syncthreads();
        prefix |= s_bin << shift;
        decided |= 255u << shift;
        remaining = s_remaining;
        __syncthreads();
    }
    const uint32_t T = prefix;            // every key above T is taken
    const uint32_t r = remaining;         // plus the first r chunks whose key equals T

    // ---- ordered compaction
    uint32_t gt_base = 0, eq_base = 0;
    for (int base = 0; base < nc; base += SEL_T) {
        const int c = base + tid;
        uint32_t gt = 0, eq = 0;
        if (c < nc) {
            const uint32_t key = ord_key(score[c]);
            gt = key > T;
            eq = key == T;
        }
        uint32_t total;
        const uint32_t ex = block_excl_scan(gt | (eq << 16), wave_tot, &total);
        const uint32_t gt_before = gt_base + (ex & 0xffffu);
        const uint32_t eq_before = eq_base + (ex >> 16);
        if (c < nc) {
            const bool take = gt || (eq && eq_before < r);
            const int32_t rank = static_cast<int32_t>(gt_before + (eq_before < r ? eq_before : r));
            if (take) sel[rank] = c;
            if (mask) mask[c] = take ? 1 : 0;
            if (slotmap) slotmap[c] = take ? rank : -1;      // what gf_fuse_pack needs to pack this selection
            if (packed_len && c == nc - 1) {
                const int64_t last_len = N - static_cast<int64_t>(nc - 1) * C;
                *packed_len = static_cast<int64_t>(k) * C - (take ? C - last_len : 0);
            }
        }
        gt_base += total & 0xffffu;
        eq_base += total >> 16;
    }
}

// The same selection with every thread holding its keys in registers: thread t owns the KPT
// consecutive chunks [t * KPT, t * KPT + KPT), reads their scores once (128-bit loads), runs the
// four radix passes on registers, and one scan over the threads' counts places its chunks in the
// ascending output.  For n_chunks <= 1024 * KPT; the time no longer grows with n_chunks.
//
// SCORE = SCORE_GIVEN: the scores are read from `score`.  Otherwise (few workers, so that one
// workgroup can read every norm) the kernel computes them first, as k_score<SCORE> would, writes
// them to `score` and goes on with them in registers: one launch instead of two.  Which chunks
// were sent is then looked up in an LDS table (chunk -> position in prev_sel) instead of a search.
constexpr int SCORE_GIVEN = -2;

struct ScoreArgs {
    const float *l1;
    const double *part;
    const float *red_l1;
    const int32_t *prev_sel;          // may be the output `sel`: read in full before the first barrier
    int32_t subs, P, k_prev;
};

template <int KPT, int SCORE>
__global__ __launch_bounds__(SEL_T) void k_select_reg(float *__restrict__ score, ScoreArgs sa, int32_t nc, int32_t k,
                                                      int32_t C, int64_t N,
                                                      int32_t *sel /* may be prev_sel */, uint8_t *__restrict__ mask,
                                                      int64_t *__restrict__ packed_len, int32_t *__restrict__ slotmap)
{
    static_assert(KPT % 4 == 0 && KPT <= 32, "counts of a thread travel in 16 bits");
    static_assert(SCORE == SCORE_GIVEN || KPT <= 16, "positions in prev_sel travel in 16 bits");
    __shared__ uint32_t hist2[2][256];      // the passes alternate between the two
    __shared__ uint32_t wave_tot[SEL_T / 64];
    __shared__ uint32_t s_bin, s_remaining;
    __shared__ int16_t sent_pos[SCORE == SCORE_GIVEN ? 1 : SEL_T * KPT];
    const int tid = threadIdx.x;
    const int base = tid * KPT;

    uint32_t key[KPT];
    if constexpr (SCORE == SCORE_GIVEN) {
        const bool vec = gf_aligned(score, 16);
#pragma unroll
        for (int i = 0; i < KPT; i += 4) {
            const int c = base + i;
            if (vec && c + 3 < nc) {
                const gf_f32x4 v = *reinterpret_cast<const gf_f32x4 *>(score + c);
                key[i] = ord_key(v.x); key[i + 1] = ord_key(v.y); key[i + 2] = ord_key(v.z); key[i + 3] = ord_key(v.w);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) key[i + j] = c + j < nc ? ord_key(score[c + j]) : 0u;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < KPT; ++i) sent_pos[base + i] = -1;
        __syncthreads();
        if (sa.prev_sel)
            for (int j = tid; j < sa.k_prev; j += SEL_T) {
                const int32_t c = sa.prev_sel[j];
                if (static_cast<uint32_t>(c) < static_cast<uint32_t>(nc)) sent_pos[c] = static_cast<int16_t>(j);
            }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < KPT; ++i) {
            const int c = base + i;
            key[i] = 0u;
            if (c < nc) {
                const int j = sent_pos[c];
                const float sc = j >= 0 ? sent_score(sa.red_l1[j], sa.P)
                                        : local_score<SCORE>(sa.l1, sa.part, sa.subs, sa.P, nc, c);
                score[c] = sc;
                key[i] = ord_key(sc);
            }
        }
    }

    // ---- key of the k-th largest score, one byte per pass
    uint32_t prefix = 0, decided = 0, remaining = static_cast<uint32_t>(k);
    if (tid < 256) hist2[0][tid] = 0;
    __syncthreads();
    for (int shift = 24, pass = 0; shift >= 0; shift -= 8, ++pass) {
        uint32_t *hist = hist2[pass & 1];
        // Neighbouring chunks often share a digit (in the first pass, sign and exponent, nearly
        // always): a thread adds each run of equal digits among its keys with one update.
        uint32_t run_digit = 0, run_len = 0;
#pragma unroll
        for (int i = 0; i < KPT; ++i) {
            if (base + i < nc && (key[i] & decided) == prefix) {
                const uint32_t d = (key[i] >> shift) & 255u;
                if (run_len && d != run_digit) { atomicAdd(&hist[run_digit], run_len); run_len = 0; }
                run_digit = d;
                ++run_len;
            }
        }
        if (run_len) atomicAdd(&hist[run_digit], run_len);
        __syncthreads();
        if (tid < 64) {
            // The first wavefront finds the bin of the remaining-th largest key on its own: lane l
            // holds bins 255 - 4l ... 252 - 4l (highest first), a scan over the lanes counts the keys
            // in higher bins.
            uint32_t cnt[4], four = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) { cnt[j] = hist[255 - 4 * tid - j]; four += cnt[j]; }
            uint32_t above = wave_incl_scan(four) - four;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (above < remaining && above + cnt[j] >= remaining) {
                    s_bin = static_cast<uint32_t>(255 - 4 * tid - j);
                    s_remaining = remaining - above;
                }
                above += cnt[j];
            }
        } else if (tid < 64 + 256) {
            hist2[(pass + 1) & 1][tid - 64] = 0;                     // meanwhile: the next pass's histogram
        }
        __syncthreads();
        prefix |= s_bin << shift;
        decided |= 255u << shift;
        remaining = s_remaining;
    }
    const uint32_t T = prefix;            // every key above T is taken
    const uint32_t r = remaining;         // plus the first r chunks whose key equals T

    // ---- ordered compaction: one scan over the threads' counts
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int i = 0; i < KPT; ++i)
        if (base + i < nc) { gt += key[i] > T; eq += key[i] == T; }
    uint32_t total;
    const uint32_t ex = block_excl_scan(gt | (eq << 16), wave_tot, &total);
    uint32_t gt_before = ex & 0xffffu, eq_before = ex >> 16;
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const int c = base + i;
        if (c < nc) {
            const bool g = key[i] > T, e = key[i] == T;
            const bool take = g || (e && eq_before < r);
            const int32_t rank = static_cast<int32_t>(gt_before + (eq_before < r ? eq_before : r));
            if (take) sel[rank] = c;
            if (mask) mask[c] = take ? 1 : 0;
            if (slotmap) slotmap[c] = take ? rank : -1;
            if (packed_len && c == nc - 1) {
                const int64_t last_len = N - static_cast<int64_t>(nc - 1) * C;
                *packed_len = static_cast<int64_t>(k) * C - (take ? C - last_len : 0);
            }
            gt_before += g;
            eq_before += e;
        }
    }
}

}  // namespace

extern "C" gf_status gf_chunk_score_select(const gf_plan *pl, const float *chunk_l1,
                                           const float *reduced_l1, const int32_t *prev_sel, int32_t k_prev,
                                           int32_t k, float *scores, int32_t *sel_idx, uint8_t *mask,
                                           int64_t *packed_len, void *workspace, gf_stream stream)
{
    if (!pl || !sel_idx) return GF_EINVAL;
    if (pl->chunk == 0 || k < 1 || k > pl->n_chunks) return GF_EINVAL;
    if (prev_sel && (!reduced_l1 || k_prev < 1 || k_prev > pl->n_chunks)) return GF_EINVAL;
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return GF_EINVAL;
    // the workspace holds the score vector when the caller does not want it, the norms when
    // gf_fuse_pack left them there, and receives the slot map of the new selection
    if ((!scores || !chunk_l1) && !workspace) return GF_EINVAL;
    char *ws = static_cast<char *>(workspace);
    if (!scores) scores = reinterpret_cast<float *>(ws + gf_ws_scores_off(pl));
    const double *part = chunk_l1 ? nullptr : reinterpret_cast<const double *>(ws + gf_ws_l1part_off(pl));
    int32_t *slotmap = ws ? reinterpret_cast<int32_t *>(ws + gf_ws_slotmap_off()) : nullptr;
    if (!pl->on_device) return GF_ESTATE;
    GF_CHECK_DEVICE(pl);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int32_t nc = pl->n_chunks;

    const int32_t subs = gf_fuse_subs(pl);
    const ScoreArgs sa{chunk_l1, part, reduced_l1, prev_sel, subs, pl->P, k_prev};
    // few workers and few chunks: the selecting workgroup computes the scores itself
    const bool one_launch = nc <= SEL_T * 8 && static_cast<int64_t>(pl->P) * (chunk_l1 ? 1 : subs) <= 8;
#define GF_SELECT(K, S) hipLaunchKernelGGL((k_select_reg<K, S>), dim3(1), dim3(SEL_T), 0, st, scores, sa, nc, k, \
                                           pl->chunk, pl->N, sel_idx, mask, packed_len, slotmap)
    if (one_launch) {
        if (nc <= SEL_T * 4) { if (chunk_l1) GF_SELECT(4, -1); else GF_SELECT(4, 0); }
        else                 { if (chunk_l1) GF_SELECT(8, -1); else GF_SELECT(8, 0); }
        GF_LAUNCH_CHECK();
        return GF_OK;
    }
    const dim3 grid((nc + GF_BLOCK - 1) / GF_BLOCK), block(GF_BLOCK);
#define GF_SCORE(S) hipLaunchKernelGGL(k_score<S>, grid, block, 0, st, chunk_l1, part, subs, pl->P, nc, reduced_l1, \
                                       prev_sel, k_prev, scores)
    if (chunk_l1) GF_SCORE(-1);
    else if (subs == 1) GF_SCORE(1);
    else if (subs == 2) GF_SCORE(2);
    else if (subs == 3) GF_SCORE(3);
    else if (subs == 4) GF_SCORE(4);
    else GF_SCORE(0);
#undef GF_SCORE
    GF_LAUNCH_CHECK();
    if (nc <= SEL_T * 4) GF_SELECT(4, SCORE_GIVEN);
    else if (nc <= SEL_T * 8) GF_SELECT(8, SCORE_GIVEN);
    else if (nc <= SEL_T * 16) GF_SELECT(16, SCORE_GIVEN);
    else if (nc <= SEL_T * 32) GF_SELECT(32, SCORE_GIVEN);
    else
        hipLaunchKernelGGL(k_select, dim3(1), dim3(SEL_T), 0, st,
                           scores, nc, k, pl->chunk, pl->N, sel_idx, mask, packed_len, slotmap);
#undef GF_SELECT
    GF_LAUNCH_CHECK();
    return GF_OK;
}
