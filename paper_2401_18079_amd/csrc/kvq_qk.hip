// Attention scores against the quantized, pre-RoPE Key cache (paper Sec. 3.2, 3.7, App. "RoPE
// Equation", App. "Kernel Implementation Details"): dense look-up-table mat-vec with the rotary
// embedding applied after de-quantisation, plus the sparse outlier mat-vec, merged in one kernel.
//
// Design (gfx950).  RoPE rotates channel i with channel i+64, so for one (token n, query head) the
// contribution of that channel pair is   A cos(n theta_i) + B sin(n theta_i)   with
//     A = q_i k_i + q_{i+64} k_{i+64},   B = q_{i+64} k_i - q_i k_{i+64},   k_c = s_c lut[code_c] + z_c.
// A and B depend on the token only through the two codes, which the storage format keeps side by
// side in one 2b-bit field.  Each workgroup therefore builds, per query head and channel pair, a
// table of (A,B) for every code pair in LDS (fp16 pairs, query, scale and zero-point folded in), and
// the hot loop per (token, head, pair) is: extract a field, one LDS gather, two mixed-precision FMAs
// with the fp32 cos/sin of the token's angle.  cos/sin are computed once per (token, pair) and
// shared by all query heads the workgroup handles.  Lanes are tokens; a wavefront reads 1 KiB of
// contiguous codes per load instruction.  For 4-bit codes the joint table would be 256 entries, so
// A and B are split into a part indexed by each code (two 16-entry gathers).
#include <utility>
#include "kvq_common.hpp"

namespace {

template <int BITS>
struct QkCfg {
    static constexpr bool JOINT = BITS <= 3;
    static constexpr int NE = 1 << BITS;
    static constexpr int ENTRIES = JOINT ? (1 << (2 * BITS)) : 2 * NE;   // half2 entries per (head, pair)
    static constexpr int CW = 4 * BITS;                                  // dwords per chunk
};

// Byte offset (field value * 4) of field `i` of a chunk held in registers, for a joint table.
template <int FBITS>   // field width in bits
__device__ inline uint32_t field_x4(const uint32_t *W, int i)
{
    const int bit = i * FBITS, wi = bit >> 5, sh = bit & 31;
    constexpr uint32_t M = ((1u << FBITS) - 1u) << 2;
    if (sh + FBITS <= 32) {
        if (sh >= 2) return (W[wi] >> (sh - 2)) & M;
        return (W[wi] << (2 - sh)) & M;
    }
    return __builtin_amdgcn_alignbit(W[wi + 1], W[wi], sh - 2) & M;
}

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

// PAIR_GROUP consecutive channel pairs of the dense part for one token.  Written gathers-first so
// that a group's LDS gathers are all in flight before the arithmetic that consumes them:
//   1. per KV head one field extraction per pair, per query head one gather,
//   2. the group's angles -> (cos, sin), shared by all query heads,
//   3. two mixed-precision FMAs per (pair, query head).
// G0 is a compile-time constant so that all register-array indices fold.
constexpr int PAIR_GROUP = 2;

template <int BITS, int QH, int R, int G0>
__device__ __forceinline__ void qk_group(const uint32_t (&W)[QH / R][QkCfg<BITS>::CW], float (&acc)[QH],
                                         const half2_t *tab, float nf, const KvqParamsHeader *hdr)
{
    using C = QkCfg<BITS>;
    constexpr int KVH = QH / R;
    constexpr int NE = C::NE;
    constexpr int ENT = C::ENTRIES;
    constexpr int NG = C::JOINT ? 1 : 2;          // gathers per (pair, query head)
    half2_t t[PAIR_GROUP][QH][NG];
#pragma unroll
    for (int p = 0; p < PAIR_GROUP; ++p) {
        constexpr int dummy = 0; (void)dummy;
        const int I = G0 * PAIR_GROUP + p;
#pragma unroll
        for (int g = 0; g < KVH; ++g) {
            uint32_t off[NG];
            if (C::JOINT) off[0] = field_x4<2 * BITS>(W[g], I);
            else { off[0] = field_x4<BITS>(W[g], 2 * I); off[NG - 1] = field_x4<BITS>(W[g], 2 * I + 1); }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int qh = g * R + r;
                const uint8_t *tb = (const uint8_t *)(tab + (qh * 64 + I) * ENT);
#pragma unroll
                for (int k = 0; k < NG; ++k) t[p][qh][k] = *(const half2_t *)(tb + k * NE * 4 + off[k]);
            }
        }
    }
    float cs[PAIR_GROUP], sn[PAIR_GROUP];
#pragma unroll
    for (int p = 0; p < PAIR_GROUP; ++p) {
        const int I = G0 * PAIR_GROUP + p;
        const float rev = rope_rev(nf, hdr->rope_vh[I], hdr->rope_vl[I]);
        cs[p] = __builtin_amdgcn_cosf(rev);
        sn[p] = __builtin_amdgcn_sinf(rev);
    }
#pragma unroll
    for (int p = 0; p < PAIR_GROUP; ++p)
#pragma unroll
        for (int qh = 0; qh < QH; ++qh)
#pragma unroll
            for (int k = 0; k < NG; ++k) {
                acc[qh] = __builtin_fmaf((float)t[p][qh][k].x, cs[p], acc[qh]);
                acc[qh] = __builtin_fmaf((float)t[p][qh][k].y, sn[p], acc[qh]);
            }
    // Pin the accumulators: an empty asm that "modifies" them and clobbers memory keeps the compiler
    // from hoisting later groups' gathers above this point (register pressure) or sinking this
    // group's arithmetic below later gathers.
#pragma unroll
    for (int qh = 0; qh < QH; ++qh) asm volatile("" : "+v"(acc[qh]) : : "memory");
}

template <int BITS, int QH, int R, int... G>
__device__ __forceinline__ void qk_all_pairs(std::integer_sequence<int, G...>,
                                             const uint32_t (&W)[QH / R][QkCfg<BITS>::CW], float (&acc)[QH],
                                             const half2_t *tab, float nf, const KvqParamsHeader *hdr)
{
    (qk_group<BITS, QH, R, G>(W, acc, tab, nf, hdr), ...);
}

template <int BITS, int QH, int R, int NT>
__global__ __launch_bounds__(NT) void kvq_qk_kernel(const void *__restrict__ params, int D, int n_kv_heads,
                                                    int64_t cap, int64_t L, const uint8_t *__restrict__ k_codes,
                                                    const uint32_t *__restrict__ k_ptr,
                                                    const uint16_t *__restrict__ k_idx,
                                                    const uint16_t *__restrict__ k_val,
                                                    const float *__restrict__ q_rot, float scale,
                                                    float *__restrict__ scores, int64_t ld, int tiles_per_wg)
{
    using C = QkCfg<BITS>;
    constexpr int KVH = QH / R;
    constexpr int NE = C::NE;
    constexpr int ENT = C::ENTRIES;
    // Statically sized LDS (up to 132 KiB of the 160 KiB a gfx950 workgroup may use): with a known base
    // address the table offsets fold into the gathers' immediate offsets.
    __shared__ __attribute__((aligned(16))) half2_t tab[QH * 64 * ENT];   // [QH][64][ENT]
    __shared__ float qs[QH * 128];                                        // query * scale
    __shared__ float2_t rope[64];                                         // (vh, vl)
    __shared__ float hmax[QH];                                            // table magnitude per head
    const KvqParamsView pv = kvq_params_view(params, D);
    const int tid = threadIdx.x;
    const int q0 = blockIdx.y * QH;
    const int kv0 = q0 / R;

    // ---- stage query, rope constants ------------------------------------------------------
    for (int j = tid; j < QH * 128; j += NT) qs[j] = q_rot[(int64_t)q0 * 128 + j] * scale;
    if (tid < 64) rope[tid] = float2_t{pv.hdr->rope_vh[tid], pv.hdr->rope_vl[tid]};
    if (tid < QH) hmax[tid] = 0.0f;
    __syncthreads();

    // ---- build the (A,B) tables -----------------------------------------------------------
    // pass 0 finds the largest magnitude per query head, pass 1 stores entries scaled by a power
    // of two so that fp16 neither overflows nor loses small heads to subnormals.
    float lut[NE];
#pragma unroll
    for (int j = 0; j < NE; ++j) lut[j] = pv.hdr->lut_k[j];
    for (int pass = 0; pass < 2; ++pass) {
        for (int e = tid; e < QH * 64 * ENT; e += NT) {
            const int qh = e / (64 * ENT), i = (e / ENT) & 63, f = e % ENT;
            const int ch = (kv0 + qh / R) * 128 + i;
            const float qa = qs[qh * 128 + i], qb = qs[qh * 128 + i + 64];
            float a, b;
            if (C::JOINT) {
                float klo = 0.f, khi = 0.f;
#pragma unroll
                for (int j = 0; j < NE; ++j) {
                    if ((f & (NE - 1)) == j) klo = __builtin_fmaf(pv.s[ch], lut[j], pv.z[ch]);
                    if ((f >> BITS) == j) khi = __builtin_fmaf(pv.s[ch + 64], lut[j], pv.z[ch + 64]);
                }
                a = qa * klo + qb * khi;
                b = qb * klo - qa * khi;
            } else {
                const int code = f & (NE - 1), upper = f >> BITS;   // [0,NE): lower channel, [NE,2NE): upper
                float k = 0.f;
#pragma unroll
                for (int j = 0; j < NE; ++j)
                    if (code == j) k = __builtin_fmaf(pv.s[ch + 64 * upper], lut[j], pv.z[ch + 64 * upper]);
                a = upper ? qb * k : qa * k;
                b = upper ? -qa * k : qb * k;
            }
            if (pass == 0) {
                float m = fmaxf(__builtin_fabsf(a), __builtin_fabsf(b));
                atomicMax((unsigned int *)&hmax[qh], __float_as_uint(m));   // non-negative floats order as uints
            } else {
                // scale so the largest entry of the head lands in [2^12, 2^13)
                int ex;
                (void)__builtin_frexpf(hmax[qh], &ex);
                const float up = __builtin_ldexpf(1.0f, 13 - ex);
                tab[e] = half2_t{(half_t)(a * up), (half_t)(b * up)};
            }
        }
        __syncthreads();
    }
    float down[QH];
#pragma unroll
    for (int qh = 0; qh < QH; ++qh) {
        int ex;
        (void)__builtin_frexpf(hmax[qh], &ex);
        down[qh] = (hmax[qh] > 0.f) ? __builtin_ldexpf(1.0f, ex - 13) : 0.f;
    }

    // ---- token tiles ------------------------------------------------------------------------
    const int64_t tile0 = (int64_t)blockIdx.x * tiles_per_wg;
    for (int tile = 0; tile < tiles_per_wg; ++tile) {
        const int64_t n = (tile0 + tile) * NT + tid;
        if (n >= L) continue;                          // no barriers below: lanes may drop out
        uint32_t W[KVH][C::CW];
#pragma unroll
        for (int g = 0; g < KVH; ++g) {
            const uint8_t *p = k_codes + kvq_k_piece0(BITS, cap, n, kv0 + g);
#pragma unroll
            for (int j = 0; j < BITS; ++j) {
                const uint4 v = *(const uint4 *)(p + j * 1024);
                W[g][4 * j + 0] = v.x; W[g][4 * j + 1] = v.y; W[g][4 * j + 2] = v.z; W[g][4 * j + 3] = v.w;
            }
        }
        const float nf = (float)n;
        float acc[QH];
#pragma unroll
        for (int qh = 0; qh < QH; ++qh) acc[qh] = 0.f;

        // dense part
        qk_all_pairs<BITS, QH, R>(std::make_integer_sequence<int, 64 / PAIR_GROUP>{}, W, acc, tab, nf, pv.hdr);
#pragma unroll
        for (int qh = 0; qh < QH; ++qh) acc[qh] *= down[qh];

        // sparse part: this token's outliers whose channel lies in the workgroup's KV heads.
        // Entries are sorted by channel; outliers are spread evenly over channels (per-channel
        // thresholds), so the start is found by interpolation and a short walk.
        {
            const uint32_t e0 = k_ptr[n], e1 = k_ptr[n + 1];
            const uint32_t target = (uint32_t)kv0 * 128u;
            uint32_t e = e0 + (uint32_t)(((uint64_t)(e1 - e0) * (uint32_t)kv0) / (uint32_t)n_kv_heads);
            while (e > e0 && k_idx[e - 1] >= target) --e;
            while (e < e1 && k_idx[e] < target) ++e;
#pragma unroll
            for (int g = 0; g < KVH; ++g) {
                while (e < e1) {
                    const uint32_t ch = k_idx[e];
                    if ((ch >> 7) != (uint32_t)(kv0 + g)) break;
                    const float v = kvq_h2f(k_val[e]);
                    const int i = ch & 63, upper = (ch >> 6) & 1;
                    const float2_t vv = rope[i];
                    const float rev = rope_rev(nf, vv.x, vv.y);
                    const float cs = __builtin_amdgcn_cosf(rev), sn = __builtin_amdgcn_sinf(rev);
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        const int qh = g * R + r;
                        const float qa = qs[qh * 128 + i], qb = qs[qh * 128 + i + 64];
                        const float qp = upper ? (qb * cs - qa * sn) : (qa * cs + qb * sn);
                        acc[qh] = __builtin_fmaf(v, qp, acc[qh]);
                    }
                    ++e;
                }
            }
        }
#pragma unroll
        for (int qh = 0; qh < QH; ++qh) scores[(int64_t)(q0 + qh) * ld + n] = acc[qh];
    }
}

template <int BITS, int QH, int R, int NT>
kvq_status launch_qk(const kvq_cache *c, const float *q, float scale, float *scores, int64_t ld, hipStream_t s)
{
    using C = QkCfg<BITS>;
    const int D = c->n_kv_heads * KVQ_HEAD_DIM;
    const int64_t L = c->n_tokens_k;
    auto kern = kvq_qk_kernel<BITS, QH, R, NT>;
    const int groups = c->n_q_heads / QH;
    const int64_t tiles = (L + NT - 1) / NT;
    // about two workgroups per compute unit in total; each builds its tables once
    int64_t tpw = (tiles * groups + 511) / 512;
    if (tpw < 1) tpw = 1;
    if (tpw > 16) tpw = 16;
    dim3 grid((unsigned)((tiles + tpw - 1) / tpw), (unsigned)groups);
    kern<<<grid, NT, 0, s>>>(c->params, D, c->n_kv_heads, c->cap_tokens, L, c->k_codes, c->k_ptr, c->k_idx,
                               c->k_val, q, scale, scores, ld, (int)tpw);
    KVQ_HIP_CHECK(hipGetLastError());
    return KVQ_OK;
}

// Query heads per workgroup: as many as fit the LDS budget, a multiple of the GQA ratio R.
template <int BITS, int R>
kvq_status dispatch_qk(const kvq_cache *c, const float *q, float scale, float *scores, int64_t ld, hipStream_t s)
{
    constexpr int QHMAX = (BITS == 3) ? 8 : 8;
    constexpr int QH = (R > QHMAX) ? R : QHMAX;
    if (c->n_q_heads % QH == 0) return launch_qk<BITS, QH, R, 512>(c, q, scale, scores, ld, s);
    // small models (fewer query heads than the preferred group): one KV head's query heads per workgroup
    return launch_qk<BITS, R, R, 512>(c, q, scale, scores, ld, s);
}

template <int BITS>
kvq_status dispatch_qk_r(const kvq_cache *c, const float *q, float scale, float *scores, int64_t ld, hipStream_t s)
{
    switch (c->n_q_heads / c->n_kv_heads) {
    case 1: return dispatch_qk<BITS, 1>(c, q, scale, scores, ld, s);
    case 2: return dispatch_qk<BITS, 2>(c, q, scale, scores, ld, s);
    case 4: return dispatch_qk<BITS, 4>(c, q, scale, scores, ld, s);
    case 8: return dispatch_qk<BITS, 8>(c, q, scale, scores, ld, s);
    default: return KVQ_ERR_UNSUPPORTED;
    }
}

}  // namespace

extern "C" kvq_status kvq_qk_matvec(const kvq_cache *cache, const float *d_q_rot, float scale, float *d_scores,
                                    int64_t ld_scores, void *stream)
{
    kvq_status st = kvq_check_cache(cache);
    if (st != KVQ_OK) return st;
    if (!cache->loaded) return KVQ_ERR_NOT_LOADED;
    if (!d_q_rot || !d_scores || ((uintptr_t)d_q_rot & 3) || ((uintptr_t)d_scores & 3)) return KVQ_ERR_INVALID_ARG;
    if (ld_scores < cache->n_tokens_k) return KVQ_ERR_INVALID_ARG;
    if (cache->n_tokens_k == 0) return KVQ_OK;
    hipStream_t s = (hipStream_t)stream;
    switch (cache->bits) {
    case 2: return dispatch_qk_r<2>(cache, d_q_rot, scale, d_scores, ld_scores, s);
    case 3: return dispatch_qk_r<3>(cache, d_q_rot, scale, d_scores, ld_scores, s);
    default: return dispatch_qk_r<4>(cache, d_q_rot, scale, d_scores, ld_scores, s);
    }
}
