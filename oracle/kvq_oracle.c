/*
 * CPU oracle for the quantized-KV-cache decode path of KVQuant (arXiv 2401.18079).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, step-by-step
 * implementation of what the GPU library must compute, written from the paper and from the
 * storage-format specification only.  It shares no code, header, table or constant generator
 * with the HIP implementation, and nothing in the product path may call it.
 *
 * What it follows (paper sections / equations):
 *   - per-channel Key and per-token Value quantisation              : Sec. 3.1
 *   - Keys are stored before the rotary embedding; the rotation of  : Sec. 3.2, App. "RoPE
 *     position n is applied to the de-quantised Key                    Equation" (element-wise form)
 *   - one sorted 2^b-entry signpost table per layer in [-1,1],      : Sec. 3.3, App. "Kernel
 *     rescaled per vector by (scale, zero-point)                       Implementation Details"
 *   - normalise A_norm=(A-z)/s, de-quantise Q(A)=s*Q(A_norm)+z      : App. "Derivation for
 *                                                                      Quantization Error"
 *   - per-vector dense-and-sparse: upper/lower outlier thresholds,  : Sec. 3.4
 *     outliers kept in 16-bit sparse form
 *   - Key thresholds/scales fixed offline, Value thresholds/scales  : Sec. 3.6, App.
 *     found online per token (top-k)                                   "Calibration Ablations"
 *   - sparse storage appended one token at a time: one 32-bit       : App. "Kernel Implementation
 *     pointer per token, 16-bit index + 16-bit value per outlier       Details", App. "Additional
 *                                                                      Experimental Details"
 *
 * Readings taken where the paper is silent (each is listed in the design document):
 *   - the signposts of a layer's datatype are fp16 numbers, like every other stored constant of the
 *     method (App. "Kernel Implementation Details": the look-up table entries and all arithmetic of
 *     the paper's kernels are fp16; App. "Additional Experimental Details": 16-bit scale and
 *     zero-point): a table handed over in fp32 is rounded to fp16, to nearest-even, once, when it is
 *     stored (kvqo_store_lut), and every later step sees only the stored values;
 *   - nearest signpost: brute-force argmin of |x_norm - lut[j]| in fp32, ties to the smaller j;
 *   - (scale, zero) = (half-range, mid-range) of the non-outliers, each rounded to fp16;
 *   - every element gets a dense code; an outlier's sparse value is the fp16-rounded residual
 *     x - dequant(code), so dense + sparse needs no mask;
 *   - Value outliers: k_side largest and k_side smallest elements of the token's D-vector;
 *   - RoPE pairs channel i with i+d/2 inside a head, theta_i = base^(-2i/d), positions from 0;
 *   - bit layout of the packed codes: see "Storage format" below.
 *
 * Pins: tests/test_oracle_*.py check every function here against closed forms, brute force,
 * textbook special cases and values derived from the paper (storage accounting).
 *
 * Storage format (head_dim d = 128 only; H = number of KV heads; D = H*128; cap = token
 * capacity, a multiple of 128; b = bits per code):
 *   Key codes.  For token n and head h the 128 codes form a "chunk" of 16*b bytes read as a
 *   little-endian bit stream: field i (0 <= i < 64) occupies stream bits [2b*i, 2b*i+2b), its low
 *   b bits are the code of channel i, its high b bits the code of channel i+64 (the two
 *   channels RoPE rotates together).  The chunk is cut into b pieces of 16 bytes; piece j of
 *   chunk (n,h) lives at byte  h*cap*16b + (n/64)*64*16b + j*1024 + (n%64)*16.
 *   Value codes.  For token pair m = n/2, head h and channel half g (channels g*64..g*64+63)
 *   the chunk is again 16*b bytes: field j holds in its low b bits the code of token 2m,
 *   channel h*128+g*64+j, and in its high b bits the code of token 2m+1, same channel.
 *   Piece r of chunk (m,h,g) lives at byte (h*2+g)*(cap/2)*16b + (m/64)*64*16b + r*1024 + (m%64)*16.
 *   Value scale / zero-point: v_sz[n][0..1] = fp16 bits of (s_n, z_n).
 *   Sparse outliers (Keys and Values alike): ptr[cap+1] (uint32, ptr[0]=0); token n owns entries
 *   ptr[n]..ptr[n+1]-1 of idx[] (uint16 channel in [0,D), ascending) and val[] (fp16 bits).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define KVQO_HEAD_DIM 128

/* ------------------------------------------------------------------ fp16 <-> fp32 */

float kvqo_h2f(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    int32_t e = (h >> 10) & 0x1f;
    uint32_t m = h & 0x3ffu;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);                 /* zero and subnormals: m * 2^-24 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024u), e - 25);    /* (1 + m/1024) * 2^(e-15) */
    return (float)(sign ? -v : v);
}

/* Round-to-nearest-even conversion, done on the exact binary expansion of the fp32 value. */
uint16_t kvqo_f2h(float f)
{
    uint32_t bits;
    memcpy(&bits, &f, 4);
    uint16_t sign = (uint16_t)((bits >> 16) & 0x8000u);
    double a = fabs((double)f);
    if (isnan(f)) return (uint16_t)(sign | 0x7e00u);
    if (a == 0.0) return sign;
    int ex;
    (void)frexp(a, &ex);                 /* a = frac * 2^ex, frac in [0.5,1) => a in [2^(ex-1), 2^ex) */
    int e = ex - 1;                      /* unbiased exponent of a */
    if (e < -14) e = -14;                /* subnormal range shares the quantum 2^-24 */
    double quantum = ldexp(1.0, e - 10); /* spacing of fp16 numbers around a */
    double q = a / quantum;              /* exact: division by a power of two */
    double r = nearbyint(q);             /* default rounding mode: to nearest, ties to even */
    double v = r * quantum;
    if (v >= 65520.0) return (uint16_t)(sign | 0x7c00u);   /* rounds to infinity */
    /* re-encode v, which is now exactly representable */
    if (v < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)(v / ldexp(1.0, -24)));
    (void)frexp(v, &ex);
    e = ex - 1;
    uint32_t mant = (uint32_t)(v / ldexp(1.0, e - 10)) - 1024u;
    return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)mant);
}

/* ------------------------------------------------------------------ storage format */

int64_t kvqo_codes_bytes(int bits, int n_kv_heads, int64_t cap)
{
    return (int64_t)n_kv_heads * cap * 16 * bits;   /* D*bits/8 bytes per token; same for K and V */
}

/* Byte offset and bit position of stream bit `sbit` of a chunk whose first piece is at `base`. */
static void chunk_bit(int64_t base, int sbit, int64_t *byte, int *bit)
{
    int piece = sbit / 128;          /* 16-byte pieces */
    int inpiece = sbit % 128;
    *byte = base + (int64_t)piece * 1024 + inpiece / 8;
    *bit = inpiece % 8;
}

static int64_t k_chunk_base(int bits, int64_t cap, int64_t n, int h)
{
    return (int64_t)h * cap * 16 * bits + (n / 64) * 64 * 16 * bits + (n % 64) * 16;
}

static int64_t v_chunk_base(int bits, int64_t cap, int64_t m, int h, int g)
{
    return (int64_t)(h * 2 + g) * (cap / 2) * 16 * bits + (m / 64) * 64 * 16 * bits + (m % 64) * 16;
}

static void put_bits(uint8_t *buf, int64_t base, int sbit0, int nbits, unsigned value)
{
    for (int k = 0; k < nbits; ++k) {
        int64_t byte; int bit;
        chunk_bit(base, sbit0 + k, &byte, &bit);
        unsigned b = (value >> k) & 1u;
        buf[byte] = (uint8_t)((buf[byte] & ~(1u << bit)) | (b << bit));
    }
}

static unsigned get_bits(const uint8_t *buf, int64_t base, int sbit0, int nbits)
{
    unsigned v = 0;
    for (int k = 0; k < nbits; ++k) {
        int64_t byte; int bit;
        chunk_bit(base, sbit0 + k, &byte, &bit);
        v |= (unsigned)((buf[byte] >> bit) & 1u) << k;
    }
    return v;
}

void kvqo_k_put(uint8_t *buf, int bits, int64_t cap, int64_t n, int ch, unsigned code)
{
    int h = ch / KVQO_HEAD_DIM, c = ch % KVQO_HEAD_DIM;
    int field = c % 64, upper = c / 64;
    put_bits(buf, k_chunk_base(bits, cap, n, h), 2 * bits * field + upper * bits, bits, code);
}

unsigned kvqo_k_get(const uint8_t *buf, int bits, int64_t cap, int64_t n, int ch)
{
    int h = ch / KVQO_HEAD_DIM, c = ch % KVQO_HEAD_DIM;
    int field = c % 64, upper = c / 64;
    return get_bits(buf, k_chunk_base(bits, cap, n, h), 2 * bits * field + upper * bits, bits);
}

void kvqo_v_put(uint8_t *buf, int bits, int64_t cap, int64_t n, int ch, unsigned code)
{
    int h = ch / KVQO_HEAD_DIM, c = ch % KVQO_HEAD_DIM;
    int g = c / 64, field = c % 64, upper = (int)(n % 2);
    put_bits(buf, v_chunk_base(bits, cap, n / 2, h, g), 2 * bits * field + upper * bits, bits, code);
}

unsigned kvqo_v_get(const uint8_t *buf, int bits, int64_t cap, int64_t n, int ch)
{
    int h = ch / KVQO_HEAD_DIM, c = ch % KVQO_HEAD_DIM;
    int g = c / 64, field = c % 64, upper = (int)(n % 2);
    return get_bits(buf, v_chunk_base(bits, cap, n / 2, h, g), 2 * bits * field + upper * bits, bits);
}

/* codes: one code per byte, [T][D]; tokens n0..n0+T-1 */
void kvqo_pack_k(uint8_t *buf, int bits, int n_kv_heads, int64_t cap, int64_t n0, int64_t T,
                 const uint8_t *codes)
{
    int D = n_kv_heads * KVQO_HEAD_DIM;
    for (int64_t t = 0; t < T; ++t)
        for (int ch = 0; ch < D; ++ch)
            kvqo_k_put(buf, bits, cap, n0 + t, ch, codes[t * D + ch]);
}

void kvqo_unpack_k(const uint8_t *buf, int bits, int n_kv_heads, int64_t cap, int64_t n0, int64_t T,
                   uint8_t *codes)
{
    int D = n_kv_heads * KVQO_HEAD_DIM;
    for (int64_t t = 0; t < T; ++t)
        for (int ch = 0; ch < D; ++ch)
            codes[t * D + ch] = (uint8_t)kvqo_k_get(buf, bits, cap, n0 + t, ch);
}

void kvqo_pack_v(uint8_t *buf, int bits, int n_kv_heads, int64_t cap, int64_t n0, int64_t T,
                 const uint8_t *codes)
{
    int D = n_kv_heads * KVQO_HEAD_DIM;
    for (int64_t t = 0; t < T; ++t)
        for (int ch = 0; ch < D; ++ch)
            kvqo_v_put(buf, bits, cap, n0 + t, ch, codes[t * D + ch]);
}

void kvqo_unpack_v(const uint8_t *buf, int bits, int n_kv_heads, int64_t cap, int64_t n0, int64_t T,
                   uint8_t *codes)
{
    int D = n_kv_heads * KVQO_HEAD_DIM;
    for (int64_t t = 0; t < T; ++t)
        for (int ch = 0; ch < D; ++ch)
            codes[t * D + ch] = (uint8_t)kvqo_v_get(buf, bits, cap, n0 + t, ch);
}

/* ------------------------------------------------------------------ quantisation */

/*
 * Store a layer's signpost table (Sec. 3.3; App. "Kernel Implementation Details": fp16 table
 * entries): each of the n_entries fp32 signposts is rounded to the nearest fp16 number (ties to
 * even) and kept as that number's fp32 value.  Rounding is monotone, so a sorted table stays sorted
 * (neighbours may become equal; the tie rule of kvqo_nearest then picks the smaller index).
 */
void kvqo_store_lut(const float *lut_in, int n_entries, float *lut_stored)
{
    for (int j = 0; j < n_entries; ++j) lut_stored[j] = kvqo_h2f(kvqo_f2h(lut_in[j]));
}

/* Nearest signpost by brute force in fp32; ties go to the smaller index. */
int kvqo_nearest(const float *lut, int n_entries, float xn)
{
    int best = 0;
    float bestd = fabsf(xn - lut[0]);
    for (int j = 1; j < n_entries; ++j) {
        float dj = fabsf(xn - lut[j]);
        if (dj < bestd) { bestd = dj; best = j; }
    }
    return best;
}

/* One element: normalise with (s,z), pick the code, return the de-quantised value. */
static int quantize_element(float x, float s, float z, const float *lut, int n_entries, float *deq)
{
    float rinv = 1.0f / s;
    float diff = x - z;
    float xn = diff * rinv;
    int code = kvqo_nearest(lut, n_entries, xn);
    *deq = fmaf(s, lut[code], z);
    return code;
}

/*
 * Keys, per channel (Sec. 3.1, 3.4, 3.6): thresholds lo/hi, scale s and zero-point z are given
 * per channel (fp16 bits).  x: fp16 bits [T][D].  Outputs: codes [T][D] (one per byte),
 * cnt[T] outliers per token, and the outliers of all T tokens concatenated in (token, ascending
 * channel) order in idx/val (at most max_nnz; the return value is the total number found).
 */
int64_t kvqo_quantize_k(const uint16_t *x, int64_t T, int D, int bits, const float *lut,
                        const uint16_t *s, const uint16_t *z, const uint16_t *lo, const uint16_t *hi,
                        uint8_t *codes, uint32_t *cnt, uint16_t *idx, uint16_t *val, int64_t max_nnz)
{
    int n_entries = 1 << bits;
    int64_t total = 0;
    for (int64_t t = 0; t < T; ++t) {
        uint32_t c_t = 0;
        for (int c = 0; c < D; ++c) {
            float xv = kvqo_h2f(x[t * D + c]);
            float deq;
            int code = quantize_element(xv, kvqo_h2f(s[c]), kvqo_h2f(z[c]), lut, n_entries, &deq);
            codes[t * D + c] = (uint8_t)code;
            if (xv < kvqo_h2f(lo[c]) || xv > kvqo_h2f(hi[c])) {
                if (total < max_nnz) {
                    idx[total] = (uint16_t)c;
                    val[total] = kvqo_f2h(xv - deq);
                }
                ++total;
                ++c_t;
            }
        }
        cnt[t] = c_t;
    }
    return total;
}

typedef struct { float v; int i; } val_idx;

static int cmp_desc(const void *a, const void *b)
{
    const val_idx *p = (const val_idx *)a, *q = (const val_idx *)b;
    if (p->v > q->v) return -1;
    if (p->v < q->v) return 1;
    return (p->i > q->i) - (p->i < q->i);      /* equal values: smaller index first */
}

static int cmp_asc(const void *a, const void *b)
{
    const val_idx *p = (const val_idx *)a, *q = (const val_idx *)b;
    if (p->v < q->v) return -1;
    if (p->v > q->v) return 1;
    return (p->i > q->i) - (p->i < q->i);
}

/*
 * Values, per token (Sec. 3.1, 3.4, 3.6): for each token the k_side largest elements are the
 * upper outliers (order: value descending, then index ascending), the k_side smallest of the
 * remaining elements are the lower outliers (value ascending, then index ascending).  The rest
 * define mx, mn; zero-point = fp16((mx+mn)/2), scale = fp16((mx-mn)/2) (scale 0 -> 1).
 * All D elements get a code; outliers additionally get a sparse residual.
 * Outputs as kvqo_quantize_k plus sz[T][2] = fp16 bits of (scale, zero-point).
 * Returns total outliers, or -1 if 2*k_side >= D.
 */
int64_t kvqo_quantize_v(const uint16_t *x, int64_t T, int D, int bits, const float *lut, int k_side,
                        uint16_t *sz, uint8_t *codes, uint32_t *cnt, uint16_t *idx, uint16_t *val,
                        int64_t max_nnz)
{
    if (2 * k_side >= D) return -1;
    int n_entries = 1 << bits;
    val_idx *w = (val_idx *)malloc(sizeof(val_idx) * (size_t)D);
    uint8_t *is_out = (uint8_t *)malloc((size_t)D);
    int64_t total = 0;
    for (int64_t t = 0; t < T; ++t) {
        memset(is_out, 0, (size_t)D);
        for (int c = 0; c < D; ++c) { w[c].v = kvqo_h2f(x[t * D + c]); w[c].i = c; }
        qsort(w, (size_t)D, sizeof(val_idx), cmp_desc);
        for (int k = 0; k < k_side; ++k) is_out[w[k].i] = 1;
        /* the remaining D-k_side elements, smallest first */
        qsort(w + k_side, (size_t)(D - k_side), sizeof(val_idx), cmp_asc);
        for (int k = 0; k < k_side; ++k) is_out[w[k_side + k].i] = 1;
        float mx = -INFINITY, mn = INFINITY;
        for (int c = 0; c < D; ++c) {
            if (is_out[c]) continue;
            float xv = kvqo_h2f(x[t * D + c]);
            if (xv > mx) mx = xv;
            if (xv < mn) mn = xv;
        }
        float sum = mx + mn, dif = mx - mn;
        uint16_t zb = kvqo_f2h(sum * 0.5f);
        uint16_t sb = kvqo_f2h(dif * 0.5f);
        float sf = kvqo_h2f(sb), zf = kvqo_h2f(zb);
        if (sf == 0.0f) { sf = 1.0f; sb = 0x3c00u; }
        sz[t * 2 + 0] = sb;
        sz[t * 2 + 1] = zb;
        uint32_t c_t = 0;
        for (int c = 0; c < D; ++c) {
            float xv = kvqo_h2f(x[t * D + c]);
            float deq;
            codes[t * D + c] = (uint8_t)quantize_element(xv, sf, zf, lut, n_entries, &deq);
            if (is_out[c]) {
                if (total < max_nnz) {
                    idx[total] = (uint16_t)c;
                    val[total] = kvqo_f2h(xv - deq);
                }
                ++total;
                ++c_t;
            }
        }
        cnt[t] = c_t;
    }
    free(w);
    free(is_out);
    return total;
}

/* ------------------------------------------------------------------ reconstruction */

/* khat[t][c] = fmaf(s_c, lut[code], z_c) + sum of the sparse values stored at (n0+t, c). */
void kvqo_reconstruct_k(const uint8_t *kbuf, int bits, int n_kv_heads, int64_t cap, const float *lut,
                        const uint16_t *s, const uint16_t *z, const uint32_t *ptr,
                        const uint16_t *idx, const uint16_t *val, int64_t n0, int64_t T, double *khat)
{
    int D = n_kv_heads * KVQO_HEAD_DIM;
    for (int64_t t = 0; t < T; ++t) {
        int64_t n = n0 + t;
        for (int c = 0; c < D; ++c) {
            unsigned code = kvqo_k_get(kbuf, bits, cap, n, c);
            khat[t * D + c] = (double)fmaf(kvqo_h2f(s[c]), lut[code], kvqo_h2f(z[c]));
        }
        for (uint32_t e = ptr[n]; e < ptr[n + 1]; ++e)
            khat[t * D + idx[e]] += (double)kvqo_h2f(val[e]);
    }
}

void kvqo_reconstruct_v(const uint8_t *vbuf, int bits, int n_kv_heads, int64_t cap, const float *lut,
                        const uint16_t *sz, const uint32_t *ptr, const uint16_t *idx,
                        const uint16_t *val, int64_t n0, int64_t T, double *vhat)
{
    int D = n_kv_heads * KVQO_HEAD_DIM;
    for (int64_t t = 0; t < T; ++t) {
        int64_t n = n0 + t;
        float sf = kvqo_h2f(sz[n * 2 + 0]), zf = kvqo_h2f(sz[n * 2 + 1]);
        for (int c = 0; c < D; ++c) {
            unsigned code = kvqo_v_get(vbuf, bits, cap, n, c);
            vhat[t * D + c] = (double)fmaf(sf, lut[code], zf);
        }
        for (uint32_t e = ptr[n]; e < ptr[n + 1]; ++e)
            vhat[t * D + idx[e]] += (double)kvqo_h2f(val[e]);
    }
}

/* ------------------------------------------------------------------ RoPE */

/*
 * Rotary embedding of one head vector at position n (element-wise form of the RoPE appendix):
 * channel i is paired with i+d/2, theta_i = base^(-2i/d) for i = 0..d/2-1,
 *   y[i]     = x[i] cos(n theta_i) - x[i+d/2] sin(n theta_i)
 *   y[i+d/2] = x[i+d/2] cos(n theta_i) + x[i] sin(n theta_i).
 */
void kvqo_rope(const double *x, int d, int64_t n, double base, double *y)
{
    int half = d / 2;
    for (int i = 0; i < half; ++i) {
        double theta = pow(base, -2.0 * (double)i / (double)d);
        double phi = (double)n * theta;
        double c = cos(phi), sn = sin(phi);
        y[i] = x[i] * c - x[i + half] * sn;
        y[i + half] = x[i + half] * c + x[i] * sn;
    }
}

/* ------------------------------------------------------------------ mat-vecs */

/*
 * scores[h][n] = scale * sum_c q[h][c] * RoPE_n(khat[n][kvhead(h)])[c],  0 <= n < L.
 * q: fp32 [n_q_heads][128], already rotated to its own position by the caller.
 * Query head h reads KV head h / (n_q_heads / n_kv_heads).  Double accumulation, fp32 result.
 * Attention-sink-aware quantization (paper Sec. 3.5): the first n_sink tokens are kept in fp16;
 * for them khat[n] is the stored pre-RoPE fp16 Key sink_k[n][D] itself (their codes are ignored).
 */
void kvqo_qk(const uint8_t *kbuf, int bits, int n_kv_heads, int n_q_heads, int64_t cap, int64_t L,
             const float *lut, const uint16_t *s, const uint16_t *z, const uint32_t *ptr,
             const uint16_t *idx, const uint16_t *val, const float *q, float scale, double rope_base,
             float *scores, int64_t ld, int64_t n_sink, const uint16_t *sink_k)
{
    const int d = KVQO_HEAD_DIM;
    int D = n_kv_heads * d;
    int group = n_q_heads / n_kv_heads;
#pragma omp parallel
    {
        double *khat = (double *)malloc(sizeof(double) * (size_t)D);
        double *krot = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(static)
        for (int64_t n = 0; n < L; ++n) {
            if (n < n_sink)
                for (int c = 0; c < D; ++c) khat[c] = (double)kvqo_h2f(sink_k[n * D + c]);
            else
                kvqo_reconstruct_k(kbuf, bits, n_kv_heads, cap, lut, s, z, ptr, idx, val, n, 1, khat);
            for (int hk = 0; hk < n_kv_heads; ++hk) {
                kvqo_rope(khat + hk * d, d, n, rope_base, krot);
                for (int j = 0; j < group; ++j) {
                    int h = hk * group + j;
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c) acc += (double)q[h * d + c] * krot[c];
                    scores[h * ld + n] = (float)((double)scale * acc);
                }
            }
        }
        free(khat);
        free(krot);
    }
}

/* probs[h][n] = exp(scores[h][n] - max_h) / sum_n exp(...), double inside, fp32 out. */
void kvqo_softmax(const float *scores, int n_q_heads, int64_t L, int64_t ld_in, float *probs,
                  int64_t ld_out)
{
    for (int h = 0; h < n_q_heads; ++h) {
        double mx = -INFINITY;
        for (int64_t n = 0; n < L; ++n)
            if ((double)scores[h * ld_in + n] > mx) mx = (double)scores[h * ld_in + n];
        double sum = 0.0;
        for (int64_t n = 0; n < L; ++n) sum += exp((double)scores[h * ld_in + n] - mx);
        for (int64_t n = 0; n < L; ++n)
            probs[h * ld_out + n] = (float)(exp((double)scores[h * ld_in + n] - mx) / sum);
    }
}

/*
 * out[h][c] = sum_n probs[h][n] * vhat[n][kvhead(h)*128 + c], double accumulation, fp32 result.
 * The first n_sink tokens are kept in fp16 (paper Sec. 3.5): vhat[n] = sink_v[n][D] for them.
 */
void kvqo_pv(const uint8_t *vbuf, int bits, int n_kv_heads, int n_q_heads, int64_t cap, int64_t L,
             const float *lut, const uint16_t *sz, const uint32_t *ptr, const uint16_t *idx,
             const uint16_t *val, const float *probs, int64_t ld, float *out, int64_t n_sink,
             const uint16_t *sink_v)
{
    const int d = KVQO_HEAD_DIM;
    int D = n_kv_heads * d;
    int group = n_q_heads / n_kv_heads;
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
    double *acc_all = (double *)calloc((size_t)nthreads * (size_t)n_q_heads * d, sizeof(double));
#pragma omp parallel
    {
        int tid = 0;
#ifdef _OPENMP
        tid = omp_get_thread_num();
#endif
        double *acc = acc_all + (size_t)tid * (size_t)n_q_heads * d;
        double *vhat = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(static)
        for (int64_t n = 0; n < L; ++n) {
            if (n < n_sink)
                for (int c = 0; c < D; ++c) vhat[c] = (double)kvqo_h2f(sink_v[n * D + c]);
            else
                kvqo_reconstruct_v(vbuf, bits, n_kv_heads, cap, lut, sz, ptr, idx, val, n, 1, vhat);
            for (int h = 0; h < n_q_heads; ++h) {
                int hk = h / group;
                double p = (double)probs[h * ld + n];
                for (int c = 0; c < d; ++c) acc[h * d + c] += p * vhat[hk * d + c];
            }
        }
        free(vhat);
    }
    for (int i = 0; i < n_q_heads * d; ++i) {
        double sum = 0.0;
        for (int t = 0; t < nthreads; ++t) sum += acc_all[(size_t)t * (size_t)n_q_heads * d + i];
        out[i] = (float)sum;
    }
    free(acc_all);
}

/* ------------------------------------------------------------------ threading control */

void kvqo_set_threads(int n)
{
#ifdef _OPENMP
    omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int kvqo_get_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
