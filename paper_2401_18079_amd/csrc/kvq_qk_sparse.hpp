// The balanced sparse Key kernel as device code, its launch plan, and the one-token pass that
// kvq_decode_step's first launch runs for the token it has just appended.  Included by the
// translation units of kvq_qk_matvec and of the appends.
#pragma once
#include "kvq_common.hpp"

namespace {

// Angle of channel pair i at position n, in revolutions, reduced to about [0,1): n*theta_i/(2 pi)
// from a two-float split of theta_i/(2 pi); the product's rounding error is recovered with an FMA,
// so the result is good to ~1e-7 revolutions for n up to 2^24.
__device__ inline float rope_rev(float nf, float vh, float vl)
{
    float p = nf * vh;
    float e = __builtin_fmaf(nf, vh, -p);
    float t = __builtin_fmaf(nf, vl, e);
    return __builtin_amdgcn_fractf(p) + t;
}

// Sparse Key outliers, balanced (paper App. "Kernel Implementation Details": equal non-zeros per
// thread): lanes are outlier entries.  Every wavefront works on its own: it owns a run of consecutive
// tokens and walks it TW tokens at a time (8, or 32 when outliers are few: see launch_qk_sparse).  A sub-range's pointers sit in one register (lane j:
// token j), so the token of an entry is a wavefront-uniform cursor plus the number of token starts
// among the 64 entries of the batch, found with scalar reads of that register.  The query is
// rotated instead of the Key (by linearity  <q, R_n (v e_c)> = v (R_n^T q)_c ) and
// scale * v * (R_n^T q)_c is accumulated into the wavefront's private LDS tile [query head][token]
// (fixed-point integer atomics: LDS floating-point atomics are an order of magnitude slower here),
// which is then written to the score buffer; the dense kernel, launched afterwards, adds its part.
// The only workgroup-wide barrier follows the staging of the scaled query.
// Row length of the LDS tile for sub-ranges of TW tokens: one token's outliers hit the same column of
// many rows, and an odd row length spreads that column over all LDS banks.
__host__ __device__ constexpr int qs_row(int tw) { return tw + 1; }
constexpr int QS_U = 6;               // 64-entry batches in flight per wavefront

__host__ __device__ constexpr int qs_wave_lds_bytes(int n_q_heads, int tw)
{
    // sums, per-pair angles, and for long sub-ranges the 64 slots of kvq_sparse_token_scan
    return ((n_q_heads * qs_row(tw) * 8 + 15) & ~15) + 64 * 8 + (tw > 8 ? 64 * 4 : 0);
}

// The work of workgroup `bx` of the sparse Key kernel (a device function: the kernel of kvq_qk_matvec
// calls it with its block index, the first launch of kvq_decode_step with its block index less the
// workgroups that append the new token there).
template <int R, int QS_TW, class SP>
__device__ __forceinline__ void qk_sparse_body(const int bx, const void *__restrict__ params, int D, int n_q_heads,
                                               int64_t L, const uint32_t *__restrict__ k_ptr, const SP ksp,
                                               uint32_t nnz_cap, const float *__restrict__ q_rot, float scale,
                                               float *__restrict__ scores, int64_t ld, int64_t tokens_per_wave)
{
    constexpr int QS_ROW = qs_row(QS_TW);
    extern __shared__ __attribute__((aligned(16))) float sparse_dyn[];
    const KvqParamsView pv = kvq_params_view(params, D);
    const int tid = threadIdx.x, lane = tid & 63, n_waves = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // scalar: loop bounds below are uniform
    float *qs = sparse_dyn;                                                     // [n_q_heads][128], scaled query
    char *mine = (char *)(sparse_dyn + n_q_heads * 128) + (size_t)wave * qs_wave_lds_bytes(n_q_heads, QS_TW);
    unsigned long long *S = (unsigned long long *)mine;                  // [n_q_heads][QS_ROW] 2^32-scaled sums
    // [64] (angle of the pair at the sub-range's first token, theta / 2 pi)
    float2_t *ang = (float2_t *)(mine + ((n_q_heads * QS_ROW * 8 + 15) & ~15));
    uint32_t *slots = (uint32_t *)(ang + 64);                            // (QS_TW > 8 only)
    const int64_t nb = ((int64_t)bx * n_waves + wave) * tokens_per_wave;
    int64_t ne = nb + tokens_per_wave;
    if (ne > L) ne = L;
    const int n_cells = n_q_heads * QS_TW;
    // the run is cut into equal sub-ranges of at most QS_TW tokens; the pointers of the next one are
    // requested while the current one is processed
    const int run = (nb < ne) ? (int)(ne - nb) : 0, n_sub = (run + QS_TW - 1) / QS_TW;
    const int sub_len = n_sub ? (run + n_sub - 1) / n_sub : 0;
    int64_t nc = nb;
    int tc = sub_len;
    uint32_t pw = 0;
    if (tc > 0) pw = k_ptr[nc + (lane < tc ? lane : tc)];
    // staging of the scaled query: its barrier comes after the first sub-range's loads are requested
    for (int j = tid; j < n_q_heads * 128; j += blockDim.x) qs[j] = q_rot[j] * scale;
    for (int j = lane; j < n_q_heads * QS_ROW; j += 64) S[j] = 0ull;
    const float my_vh = pv.hdr->rope_vh[lane], my_vl = pv.hdr->rope_vl[lane];
    bool staged = false, have_next = false;
    uint32_t chn[QS_U], vbn[QS_U];
    while (tc > 0) {
        const int64_t nc_next = nc + tc;
        const int tc_next = (int)((ne - nc_next < sub_len) ? (ne - nc_next) : sub_len);
        const uint32_t e_begin = (uint32_t)__builtin_amdgcn_readfirstlane((int)pw);
        const uint32_t e_end = (uint32_t)__builtin_amdgcn_readlane((int)pw, 63);
        uint32_t chv[QS_U], vb[QS_U];
        if (e_begin < e_end) {
            if (have_next) {                             // requested during the previous sub-range
#pragma unroll
                for (int u = 0; u < QS_U; ++u) { chv[u] = chn[u]; vb[u] = vbn[u]; }
            } else if (e_begin + 64u * QS_U <= nnz_cap) {
                kvq_sparse_load_batch<false, QS_U>(ksp, nnz_cap, e_begin, e_end, lane, chv, vb);
            } else {
                kvq_sparse_load_batch<true, QS_U>(ksp, nnz_cap, e_begin, e_end, lane, chv, vb);
            }
        }
        // the next sub-range's entries follow this one's: request its first batch now (its end is not
        // known yet, so the whole batch is requested, which must then lie inside the arrays)
        have_next = tc_next > 0 && e_end + 64u * QS_U <= nnz_cap;
        if (have_next) kvq_sparse_load_batch<false, QS_U>(ksp, nnz_cap, e_end, 0xFFFFFFFFu, lane, chn, vbn);
        uint32_t pw_next = 0;
        if (tc_next > 0) pw_next = k_ptr[nc_next + (lane < tc_next ? lane : tc_next)];
        ang[lane] = float2_t{rope_rev((float)nc, my_vh, my_vl), my_vh};
        if (!staged) {
            __syncthreads();
            staged = true;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // Short sub-ranges: the pointers of tokens 1 .. QS_TW - 1 as scalars (lanes from tc on hold the
        // sub-range's end, which no entry reaches); an entry's token is the number of them it has
        // reached: straight-line compares instead of the walk of kvq_sparse_token, whose scalar loops
        // cost this kernel more than the arithmetic on the entries does.
        constexpr int NPJ = (QS_TW <= 8) ? QS_TW - 1 : 1;
        uint32_t pj[NPJ];
        if (QS_TW <= 8) {
#pragma unroll
            for (int j = 0; j < NPJ; ++j) pj[j] = (uint32_t)__builtin_amdgcn_readlane((int)pw, j + 1);
        }
        for (uint32_t eb = e_begin; eb < e_end; eb += 64 * QS_U) {
            if (eb != e_begin) {                         // (the first batch was requested above)
                if (eb + 64u * QS_U <= nnz_cap)
                    kvq_sparse_load_batch<false, QS_U>(ksp, nnz_cap, eb, e_end, lane, chv, vb);
                else
                    kvq_sparse_load_batch<true, QS_U>(ksp, nnz_cap, eb, e_end, lane, chv, vb);
            }
#pragma unroll
            for (int u = 0; u < QS_U; ++u) {
                const uint32_t first = eb + 64u * u, e = first + (uint32_t)lane;
                if (first >= e_end) break;
                int t;
                if (QS_TW <= 8) {
                    t = 0;
#pragma unroll
                    for (int j = 0; j < NPJ; ++j) t += (e >= pj[j]) ? 1 : 0;
                } else {
                    t = kvq_sparse_token_scan(pw, tc, first, lane, slots);
                }
                if (e < e_end) {
                    const uint32_t ch = chv[u];
                    const float v = kvq_h2f((uint16_t)vb[u]);
                    const float2_t a = ang[ch & 63];
                    const float rev = __builtin_fmaf((float)t, a.y, a.x);
                    const float cs = __builtin_amdgcn_cosf(rev);
                    // (R_n^T q)_c = q_c cos + s q_{c^64} sin with s = +1 for the lower channel of the
                    // pair and -1 for the upper: fold s into the sine
                    const float sn = __builtin_bit_cast(
                        float, __builtin_bit_cast(uint32_t, __builtin_amdgcn_sinf(rev)) ^ ((ch & 64u) << 25));
                    const uint32_t cl = ch & 127u, kvh = ch >> 7;
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        const uint32_t qh = kvh * R + r;
                        const uint32_t qi = (R == 1) ? ch : qh * 128u + cl;
                        const float qp = qs[qi] * cs + qs[qi ^ 64u] * sn;
                        kvq_lds_add_fixed<0>(&S[__umul24(qh, QS_ROW) + t], v * qp);     // 24-bit multiply: full rate
                    }
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // write the tile to the score buffer and clear it for the next sub-range
        for (int j = lane; j < n_cells; j += 64) {
            const int qh = j / QS_TW, t = j % QS_TW;
            const unsigned long long x = S[qh * QS_ROW + t];
            S[qh * QS_ROW + t] = 0ull;
            if (t < tc) scores[(int64_t)qh * ld + nc + t] = kvq_from_fixed_fast<0>(x);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        nc = nc_next;
        tc = tc_next;
        pw = pw_next;
    }
    if (!staged) __syncthreads();        // a wavefront without tokens still meets the workgroup's barrier
}


// Launch plan of the sparse Key kernel for sub-ranges of `tw` tokens.  LDS: the scaled query plus one
// private slice per wavefront (and `static_lds` bytes that the kernel declares for other purposes);
// two workgroups of 16 wavefronts per CU when they fit in 77 KiB each, fewer wavefronts otherwise.
// The grid holds as many wavefronts as the chip holds at once (160 KiB of LDS and 32 wavefronts per
// compute unit), every one with the same number of tokens.
struct QkSparsePlan {
    int waves;                 // wavefronts per workgroup
    size_t lds;                // dynamic LDS bytes
    int64_t tokens_per_wave;
    unsigned grid;             // workgroups
};
inline bool qk_sparse_plan(int n_q_heads, int64_t L, int tw, size_t static_lds, QkSparsePlan &p)
{
    const int per_wave = qs_wave_lds_bytes(n_q_heads, tw);
    int waves = 16;
    while (waves > 1 && static_lds + (size_t)n_q_heads * 512 + (size_t)waves * per_wave > 78848)
        waves -= (waves > 4) ? 4 : waves / 2;
    const size_t lds = (size_t)n_q_heads * 512 + (size_t)waves * per_wave;
    if (static_lds + lds > 147456) return false;
    int wgs_per_cu = (int)(163840 / (static_lds + lds));
    if (wgs_per_cu * waves > 32) wgs_per_cu = 32 / waves;
    if (wgs_per_cu < 1) wgs_per_cu = 1;
    const int64_t resident = (int64_t)kvq_cu_count() * wgs_per_cu * waves;
    int64_t tpw = (L + resident - 1) / resident;
    if (tpw < 1) tpw = 1;
    if (tw > 8) tpw = (tpw + tw - 1) / tw * tw;          // whole sub-ranges: full cache lines of scores
    const int64_t n_waves = (L + tpw - 1) / tpw;
    p.waves = waves;
    p.lds = lds;
    p.tokens_per_wave = tpw;
    p.grid = (unsigned)((n_waves + waves - 1) / waves);
    return true;
}

}  // namespace
