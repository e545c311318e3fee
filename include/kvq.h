/*
 * kvq — decode-time attention mat-vecs against a sub-4-bit non-uniformly quantized KV cache
 * (KVQuant, arXiv 2401.18079), native for AMD MI355X (gfx950).
 *
 * C ABI.  All pointers named d_* or stored in kvq_cache are DEVICE pointers (HIP global memory,
 * e.g. torch tensors' data_ptr()); pointers named h_* are HOST pointers.  `stream` is a
 * hipStream_t passed as void* (NULL = the default stream).  Every call is asynchronous on
 * `stream` unless stated otherwise.  The library allocates and frees no device memory: the
 * caller owns every buffer, sized with the kvq_*_bytes helpers below.
 *
 * Threads: calls on different caches may be made from different host threads, except for the timing
 * aid at the end of this file; calls on one cache, or on caches that share a workspace, must not
 * overlap, on the host or on the GPU (they share the workspace and the descriptor's token counts).
 * One GPU: the device that is current when a cache's buffers are allocated.
 *
 * Supported shapes: head_dim = 128; bits in {2,3,4}; n_q_heads a multiple of n_kv_heads;
 * D = n_kv_heads*128 <= 65536; cap_tokens a multiple of 128, below 2^24.  Narrower limits of single
 * calls (they return KVQ_ERR_UNSUPPORTED beyond them): kvq_qk_matvec and kvq_attention_decode take
 * n_q_heads / n_kv_heads in {1, 2, 4, 8}; kvq_quantize_append_v and kvq_quantize_append_kv take
 * D <= 16384 (a token's vector is selected from in LDS); kvq_pv_matvec takes any ratio.
 * Inputs are finite fp16 / fp32 numbers: NaN and infinities are undefined behaviour of the method
 * (no error is raised; a cache whose Key thresholds are all -65504 / +65504 skips the sparse Key
 * kernel although an infinite Key would have been recorded as an outlier).
 *
 * Storage format (owned by this library, bit-exact and documented so that a reference
 * implementation can check it):
 *   Key codes   — per KV head a plane of cap_tokens chunks; the chunk of (token n, head h) is a
 *                 16*bits-byte little-endian bit stream of 64 fields of 2*bits bits; field i holds
 *                 the code of channel i (low bits) and of channel i+64 (high bits), the two channels
 *                 RoPE rotates together.  The chunk is stored as `bits` pieces of 16 bytes, piece j
 *                 at byte  h*cap*16*bits + (n/64)*64*16*bits + j*1024 + (n%64)*16
 *                 (tokens interleaved in blocks of 64 so a wavefront reads 1 KiB contiguous).
 *   Value codes — per (KV head h, channel half g) a plane of cap_tokens/2 chunks; the chunk of
 *                 (token pair m, h, g) has the same shape; field j holds the code of channel
 *                 h*128+g*64+j for token 2m (low bits) and 2m+1 (high bits).  Piece r at byte
 *                 (h*2+g)*(cap/2)*16*bits + (m/64)*64*16*bits + r*1024 + (m%64)*16.
 *   v_sz        — [cap_tokens][2] fp16: per-token Value scale and zero-point.
 *   Sparse outliers (Keys and Values): ptr[cap_tokens+1] uint32 with ptr[0]=0; token n owns
 *                 entries ptr[n]..ptr[n+1]-1 of idx[] (uint16 channel in [0,D), ascending) and
 *                 val[] (fp16 bits of the residual x - dequant(code)).
 *   Sink tokens — sink_k / sink_v [n_sink][D] fp16: the unquantized rows of the first n_sink tokens.
 * All cache buffers must be zero-filled before the first append (ptr[0] must be 0).
 */
#ifndef KVQ_H
#define KVQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KVQ_OK = 0,
    KVQ_ERR_INVALID_ARG = 1,   /* null / misaligned pointer, bad count, 2*k_side_v >= D, ...           */
    KVQ_ERR_UNSUPPORTED = 2,   /* bits not in {2,3,4}, head_dim != 128, ...                            */
    KVQ_ERR_CAPACITY = 3,      /* n_tokens + T > cap_tokens, or workspace too small (host-detected)    */
    KVQ_ERR_NNZ_OVERFLOW = 4,  /* reported through *d_status by the device when a sparse array is full */
    KVQ_ERR_NOT_LOADED = 5,    /* kvq_lut_load has not been called on this cache                       */
    KVQ_ERR_HIP = 6            /* a HIP runtime call failed                                            */
} kvq_status;

/*
 * One layer's cache for one sequence.  Plain data, owned by the caller, lives in HOST memory;
 * the pointers inside are DEVICE pointers, each 16-byte aligned.  A batch of independent
 * sequences is an array of these (one call per sequence).
 */
typedef struct kvq_cache {
    int32_t bits;           /* 2, 3 or 4                                                        */
    int32_t head_dim;       /* 128                                                              */
    int32_t n_kv_heads;     /* H; D = H*head_dim is the vector the method quantizes per token   */
    int32_t n_q_heads;      /* multiple of n_kv_heads; query head q reads KV head q/(Hq/H)      */
    int32_t k_side_v;       /* Value outliers kept per side (largest / smallest) of each token  */
    int32_t loaded;         /* set by kvq_lut_load (0 = not loaded)                             */
    int64_t cap_tokens;     /* multiple of 128                                                  */
    int64_t n_tokens_k;     /* tokens appended so far; advanced by kvq_quantize_append_k        */
    int64_t n_tokens_v;     /* likewise for kvq_quantize_append_v                               */
    int64_t cap_nnz_k;      /* entries in k_idx / k_val                                         */
    int64_t cap_nnz_v;      /* entries in v_idx / v_val                                         */
    float rope_base;        /* 10000 (LLaMA / Llama-2) or 500000 (Llama-3)                      */
    int32_t n_sink;         /* attention-sink tokens kept in fp16 (paper Sec. 3.5): 0..KVQ_MAX_SINK */
    void *params;           /* kvq_params_bytes() bytes, filled by kvq_lut_load                 */
    uint8_t *k_codes;       /* kvq_codes_bytes() bytes                                          */
    uint8_t *v_codes;       /* kvq_codes_bytes() bytes                                          */
    uint16_t *v_sz;         /* [cap_tokens][2] fp16 (scale, zero-point)                         */
    uint32_t *k_ptr;        /* [cap_tokens+1]                                                   */
    uint32_t *v_ptr;        /* [cap_tokens+1]                                                   */
    uint16_t *k_idx, *k_val;/* [cap_nnz_k]                                                      */
    uint16_t *v_idx, *v_val;/* [cap_nnz_v]                                                      */
    int32_t *d_status;      /* one device word: 0, or a sticky kvq_status set by a kernel       */
    void *workspace;        /* scratch for partial results, >= kvq_workspace_bytes()            */
    int64_t workspace_bytes;
    uint16_t *sink_k;       /* [n_sink][D] fp16: pre-RoPE Keys of tokens 0..n_sink-1 (NULL if 0) */
    uint16_t *sink_v;       /* [n_sink][D] fp16: Values of tokens 0..n_sink-1 (NULL if n_sink=0) */
    /* Blocked outlier storage (see below).  0: k_idx .. v_val above are flat arrays.  Otherwise they
     * are ignored and the four tables that follow list the blocks, 2^nnz_block_shift entries each.   */
    int32_t nnz_block_shift;
    int32_t reserved0;      /* 0                                                                 */
    uint16_t **k_idx_blocks, **k_val_blocks; /* DEVICE arrays [cap_nnz_k >> shift] of DEVICE pointers */
    uint16_t **v_idx_blocks, **v_val_blocks; /* DEVICE arrays [cap_nnz_v >> shift] of DEVICE pointers */
} kvq_cache;

/*
 * Blocked outlier storage (paper App. "Limitations": the sparse matrix allocated in blocks, so that
 * appending a token does not copy the entries already stored).  With nnz_block_shift = s in
 * [KVQ_NNZ_BLOCK_SHIFT_MIN, KVQ_NNZ_BLOCK_SHIFT_MAX], sparse entry e of the Keys is element
 * e & (2^s - 1) of the block k_idx_blocks[e >> s] (its index) and k_val_blocks[e >> s] (its value),
 * likewise for the Values; the entry numbering, k_ptr / v_ptr and every result are those of the flat
 * layout, which is the case of one block.  cap_nnz_k and cap_nnz_v are whole numbers of blocks
 * (at least one) and every table slot below cap_nnz >> s holds a valid block of 2^s uint16
 * (2-byte aligned is enough).  To grow, the owner allocates one more block, stores its address in
 * the next slot of the table (the tables are the caller's: size them for the largest capacity
 * wanted, 8 bytes per block) and adds 2^s to cap_nnz between two calls; nothing stored moves.
 * The library only reads the tables.  Checked on the host: shift range, capacities, table pointers
 * non-null and 8-byte aligned (INVALID_ARG); the block addresses themselves live on the device and
 * are not checked.
 */
#define KVQ_NNZ_BLOCK_SHIFT_MIN 10
#define KVQ_NNZ_BLOCK_SHIFT_MAX 30

/*
 * Attention-sink-aware quantization (paper Sec. 3.5): the first n_sink tokens of the sequence stay
 * in fp16.  The append calls still quantize them like any other token (so the packed arrays do not
 * depend on n_sink) and also copy their fp16 rows to sink_k / sink_v; kvq_qk_matvec and
 * kvq_pv_matvec use the fp16 rows for those tokens and ignore their codes and outliers.
 */
#define KVQ_MAX_SINK 4

/* Buffer sizes in bytes. */
int64_t kvq_codes_bytes(int32_t bits, int32_t n_kv_heads, int64_t cap_tokens); /* = cap*D*bits/8 */
int64_t kvq_params_bytes(int32_t n_kv_heads);
/* Scratch needed by any call on this cache with at most max_append tokens per append call. */
int64_t kvq_workspace_bytes(const kvq_cache *cache, int32_t max_append);

const char *kvq_status_string(kvq_status s);
const char *kvq_version(void);

/*
 * Stage one layer's quantization constants on the device (paper Sec. 3.3: one sorted 2^bits-entry
 * signpost table per layer for Keys and one for Values, in [-1,1]; Sec. 3.1/3.4/3.6: per-channel
 * Key scale, zero-point and lower/upper outlier thresholds calibrated offline).
 *   h_lut_k, h_lut_v : HOST fp32 [2^bits], ascending.  The signposts of the datatype are fp16 numbers
 *                      (the paper's look-up tables hold fp16 entries, App. "Kernel Implementation
 *                      Details"): each entry is rounded to the nearest fp16 number, ties to even, as
 *                      it is stored, and the appends and both mat-vecs all use the stored values
 *                      (as fp32 in the arithmetic).  Entries may become equal by the rounding; the
 *                      nearest-signpost rule then picks the smaller index.
 *   h_s_k, h_z_k, h_lo_k, h_hi_k : HOST fp16 bit patterns [D].
 * Copies synchronously from the host arrays (they may be freed on return), then runs a small
 * kernel on `stream`.  Sets cache->loaded.  Errors: INVALID_ARG, UNSUPPORTED, HIP.
 */
kvq_status kvq_lut_load(kvq_cache *cache, const float *h_lut_k, const float *h_lut_v,
                        const uint16_t *h_s_k, const uint16_t *h_z_k,
                        const uint16_t *h_lo_k, const uint16_t *h_hi_k, void *stream);
/* The value kvq_lut_load stores for a signpost x (host-only arithmetic, no GPU needed): the nearest
 * fp16 number, ties to even, as fp32; NaN if |x| >= 65520 or x is NaN (kvq_lut_load rejects those). */
float kvq_stored_signpost(float x);

/*
 * Quantize T new pre-RoPE Key vectors and append them (paper Sec. 3.1, 3.2, 3.4, 3.7; the
 * normalise / de-quantise equations of App. "Derivation for Quantization Error").  Per element:
 * x_norm = (x - z_c) * (1/s_c) in fp32, code = nearest signpost (ties to the smaller index),
 * outlier iff x < lo_c or x > hi_c; an outlier's sparse value is fp16(x - fmaf(s_c, lut[code], z_c)).
 *   d_k_new : DEVICE fp16 [T][D], row t is token n_tokens_k + t.  1 <= T <= 4096.  Any fp16-aligned
 *             address (16-byte alignment lets the outlier count of a multi-token call use wide loads).
 * Writes the packed codes, k_ptr[n+1..n+T], k_idx/k_val; advances cache->n_tokens_k by T.
 * Outliers that do not fit cap_nnz_k are dropped (highest channels of the overflowing token
 * first) and *d_status is set to KVQ_ERR_NNZ_OVERFLOW.  Host errors: INVALID_ARG, CAPACITY,
 * NOT_LOADED, HIP (nothing is launched, n_tokens_k unchanged).
 */
kvq_status kvq_quantize_append_k(kvq_cache *cache, const uint16_t *d_k_new, int32_t T, void *stream);

/*
 * Quantize T new Value vectors per token and append them (paper Sec. 3.1, 3.4, 3.6: outlier
 * thresholds and scaling found online per token).  Per token: the k_side_v largest elements
 * (value descending, then index ascending) and the k_side_v smallest of the rest (value
 * ascending, then index ascending) are outliers; mx/mn of the rest give zero = fp16((mx+mn)/2),
 * scale = fp16((mx-mn)/2) (0 -> 1); then every element is coded as for Keys with (scale, zero).
 *   d_v_new : DEVICE fp16 [T][D].  1 <= T <= 4096.
 * Writes codes, v_sz, v_ptr, v_idx/v_val; advances cache->n_tokens_v.  Errors as for Keys.
 */
kvq_status kvq_quantize_append_v(kvq_cache *cache, const uint16_t *d_v_new, int32_t T, void *stream);

/*
 * Both appends of a decode step in one call and, for the quantization itself, one kernel launch:
 * exactly kvq_quantize_append_k(cache, d_k_new, T) followed by kvq_quantize_append_v(cache, d_v_new, T)
 * (paper Sec. 3.1-3.4, 3.6 as above), with the workgroups of the two running side by side: a
 * single-token append is latency-bound and the two do not depend on each other (from 256 tokens per
 * call on, where either kernel fills the GPU alone, the two run one after the other).  The checks of both
 * calls are made before anything is launched; n_tokens_k and n_tokens_v both advance by T.
 */
kvq_status kvq_quantize_append_kv(kvq_cache *cache, const uint16_t *d_k_new, const uint16_t *d_v_new,
                                  int32_t T, void *stream);

/*
 * Attention scores against the quantized Keys, dense and sparse parts merged in one result
 * (paper Sec. 3.2 and App. "RoPE Equation": the rotation of position n is applied to the
 * de-quantised Key; App. "Kernel Implementation Details": LUT mat-vec plus sparse mat-vec):
 *   scores[q][n] = scale * sum_c q_rot[q][c] * RoPE_n(khat[n][kv(q)])[c],   0 <= n < n_tokens_k,
 *   khat[n][c] = s_c*lut_k[code] + z_c + (sparse residual at (n,c)); RoPE pairs channel i with i+64,
 *   theta_i = rope_base^(-2i/128), positions from 0.
 *   d_q_rot  : DEVICE fp32 [n_q_heads][128], already rotated to the query's own position.
 *   d_scores : DEVICE fp32 [n_q_heads][ld_scores], ld_scores >= n_tokens_k; entries n >= n_tokens_k
 *              are not touched.
 * fp32 tables and fp32 accumulation throughout.  Errors: INVALID_ARG, NOT_LOADED, UNSUPPORTED
 * (n_q_heads / n_kv_heads not in {1, 2, 4, 8}), HIP.
 */
kvq_status kvq_qk_matvec(const kvq_cache *cache, const float *d_q_rot, float scale,
                         float *d_scores, int64_t ld_scores, void *stream);

/*
 * Attention output against the quantized Values, dense and sparse parts merged (paper App.
 * "Kernel Implementation Details"):
 *   out[q][c] = sum_{n < n_tokens_v} probs[q][n] * vhat[n][kv(q)*128 + c],
 *   vhat[n][c] = s_n*lut_v[code] + z_n + (sparse residual at (n,c)).
 *   d_probs : DEVICE fp32 [n_q_heads][ld_probs];  d_out : DEVICE fp32 [n_q_heads][128].
 * fp32 accumulation in a fixed order (results are run-to-run identical).  Uses cache->workspace.
 * Range: the sparse part is summed per workgroup in 64-bit fixed point with 40 fractional bits, so
 * |sum over a workgroup's tokens of probs[q][n] * residual(n, c)| must stay below 2^23 for every
 * (q, c); with softmax weights (sum <= 1) and fp16 residuals (|r| <= 65504) it always does, with
 * arbitrary caller-made weights it is the caller's to ensure (no error is raised; the sum wraps).
 */
kvq_status kvq_pv_matvec(const kvq_cache *cache, const float *d_probs, int64_t ld_probs,
                         float *d_out, void *stream);

/*
 * One decode step's attention in a single call: kvq_qk_matvec, the softmax over the scores and
 * kvq_pv_matvec (paper Sec. 3 and App. "Kernel Implementation Details": the two mat-vecs of
 * generation-time attention with the softmax between them), without separate softmax passes over
 * the scores: the Key kernels leave per-workgroup score maxima in the cache's workspace, the Value
 * kernels weight a token by exp(score - max) as they load its score, and the final reduction
 * divides by the sum of the weights.
 *   out[q][c] = sum_n softmax_n(scores[q][.])[n] * vhat[n][kv(q)*128 + c]
 * with scores and vhat as defined for the two calls above.  Requires n_tokens_k == n_tokens_v
 * (INVALID_ARG otherwise).
 *   d_q_rot  : DEVICE fp32 [n_q_heads][128], rotated to the query's position.
 *   d_scores : DEVICE fp32 [n_q_heads][ld_scores] scratch, ld_scores >= n_tokens_k; on return it
 *              holds the raw scores (not the probabilities); entries n >= n_tokens_k untouched.
 *   d_out    : DEVICE fp32 [n_q_heads][128]; all zero when the cache is empty.
 * Uses cache->workspace (kvq_workspace_bytes covers it).  Errors as for the two mat-vecs.
 */
kvq_status kvq_attention_decode(const kvq_cache *cache, const float *d_q_rot, float scale,
                                float *d_scores, int64_t ld_scores, float *d_out, void *stream);

/*
 * One generation step of one layer for one sequence in a single call (paper Sec. 3: at every step
 * the new token's Key and Value join the cache and the query attends over all of it):
 * kvq_quantize_append_kv(cache, d_k_new, d_v_new, 1) followed by kvq_attention_decode on the cache
 * that now ends with the new token.  The cache ends up bit for bit as after that append.  For flat
 * outlier storage, D = 1024 or 4096 and caches sized for 16 or more Key outliers per token the append
 * and the sparse Key kernel over the older tokens run as workgroups of ONE launch (the append is
 * latency only and the sparse kernel needs the new token for the last score alone; the workgroup that
 * quantizes the new Key also sums the sparse part of its score): the scores and outputs then agree
 * with the two calls to rounding (sums of the same terms split at other token boundaries), not bit for
 * bit.  Every other shape runs exactly the two calls.
 *   d_k_new, d_v_new : DEVICE fp16 [D], the new token's pre-RoPE Key and its Value.
 *   d_q_rot, scale, d_scores, ld_scores, d_out : as for kvq_attention_decode; ld_scores must cover
 *   the new token too (>= n_tokens_k + 1 on entry).
 * Every host-side check of both halves is made before anything is launched, so a call that returns
 * INVALID_ARG, CAPACITY or NOT_LOADED has changed nothing; UNSUPPORTED (a shape beyond the mat-vecs'
 * limits) and HIP can come back after the append has been launched, in which case n_tokens_k and
 * n_tokens_v have advanced.
 */
kvq_status kvq_decode_step(kvq_cache *cache, const uint16_t *d_k_new, const uint16_t *d_v_new,
                           const float *d_q_rot, float scale, float *d_scores, int64_t ld_scores,
                           float *d_out, void *stream);
/* Kernel launches of the next kvq_decode_step on this cache (host arithmetic plus one query of kernel
 * attributes on the current device): 5 when the append and the sparse Key kernel share a launch, 6 when
 * the step is the two calls (5 if the thresholds admit no Key outlier: no sparse Key kernel), one more
 * with attention-sink tokens (their score kernel); copies of sink rows not counted.  -1: the descriptor is not usable for a step (the step call says why). */
int32_t kvq_decode_step_launches(const kvq_cache *cache);

/*
 * kvq_attention_decode for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels and
 * the same result, bit for bit, but the scratch (slab partials of the Value kernels, softmax
 * statistics) is a static array in the library's device image instead of cache->workspace, which is
 * ignored and may be NULL.  The array (16.2 MiB) exists once per GPU from the moment the library is
 * loaded there until the process ends; its address is looked up on the first call on each device
 * (no allocation then either).  Limit: n_q_heads <= 32 (KVQ_ERR_CAPACITY beyond; nothing is launched).
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two streams, two
 * threads) race and must be serialised by the caller.  Nothing needs clearing between calls: the
 * kernels write every slot they later read.  Arguments and other errors as kvq_attention_decode.
 */
kvq_status kvq_attention_decode_noalloc(const kvq_cache *cache, const float *d_q_rot, float scale,
                                        float *d_scores, int64_t ld_scores, float *d_out, void *stream);

/* ---- helpers beyond the calls above ------------------------------------------------------- */

/*
 * Row-wise softmax in fp32 with max subtraction: probs[q][n] = exp(x[q][n]-max_q)/sum, n < n_cols.
 * d_workspace: at least kvq_softmax_workspace_bytes(n_rows, n_cols) bytes.  In-place allowed.
 */
int64_t kvq_softmax_workspace_bytes(int32_t n_rows, int64_t n_cols);
kvq_status kvq_softmax_f32(const float *d_x, int64_t ld_x, float *d_probs, int64_t ld_probs,
                           int32_t n_rows, int64_t n_cols, void *d_workspace, int64_t workspace_bytes,
                           void *stream);

/*
 * Offline derivation of the non-uniform datatype of one Key or Value layer (paper Sec. 3.3, Eq. (1),
 * with the weighting of the appendix on per-channel scaling): Lloyd's k-means iteration in one
 * dimension for the 2^bits signposts c that minimise  sum_i w[i] * (x[i] - nearest_c(x[i]))^2.
 *   d_x_norm   : DEVICE fp32 [n], calibration activations normalised per vector to [-1, 1].
 *   d_w        : DEVICE fp32 [n], w[i] = F_ii * s_i^2 >= 0 (Fisher information times squared scale).
 *   h_signposts: HOST fp32 [2^bits]; in: initial signposts, out: the signposts after `iters`
 *                iterations, sorted ascending.  The call synchronizes the stream before returning.
 *   d_workspace: DEVICE, 256-byte aligned, at least kvq_calibrate_workspace_bytes() bytes.
 * An iteration assigns every element to its nearest signpost (fp32 distances, ties to the smaller
 * index) and moves every signpost to the weighted mean of its elements (fp64 sums in a fixed order,
 * rounded to fp32); a signpost whose elements have total weight zero stays.  Both arrays 16-byte
 * aligned, n >= 1, iters >= 0.  Errors: INVALID_ARG, UNSUPPORTED (bits), CAPACITY (workspace), HIP.
 */
/*
 * Offline per-channel calibration of the Keys of one layer (paper Sec. 3.6 and the appendix on offline
 * calibration; Sec. 3.4 for the outlier fraction): from T calibration Key vectors, per channel, the
 * lower / upper outlier thresholds (the k-th smallest / k-th largest value, k = floor(fraction/2*T+1/2)
 * per side), and zero-point (mid-range) and scale (half-range; not positive -> 1) of the values
 * strictly inside, each rounded to fp16: the four arrays kvq_lut_load takes.  fraction = 0: thresholds
 * -65504 / +65504 and the full range.
 *   d_k_cal : DEVICE fp16 [T][D], pre-RoPE.  1 <= T <= 32768, 2k < T.
 *   d_s, d_z, d_lo, d_hi : DEVICE fp16 bit patterns [D] (copy them to the host for kvq_lut_load).
 * Asynchronous on `stream`.  Errors: INVALID_ARG, UNSUPPORTED (T), HIP.
 */
kvq_status kvq_calibrate_key_channels(const uint16_t *d_k_cal, int32_t T, int32_t D, float outlier_fraction,
                                      uint16_t *d_s, uint16_t *d_z, uint16_t *d_lo, uint16_t *d_hi,
                                      void *stream);

int64_t kvq_calibrate_workspace_bytes(void);
kvq_status kvq_calibrate_nuq(const float *d_x_norm, const float *d_w, int64_t n, int32_t bits,
                             int32_t iters, float *h_signposts, void *d_workspace,
                             int64_t workspace_bytes, void *stream);

/*
 * Same-GPU fp16-cache baselines (what the quantized path is compared against):
 *   scores[q][n] = scale * sum_c q[q][c] * K16[n][kv(q)*128+c]   (K16 fp16 [L][D], already rotated)
 *   out[q][c]    = sum_n probs[q][n] * V16[n][kv(q)*128+c]
 * d_workspace for the PV baseline: kvq_fp16_pv_workspace_bytes(n_q_heads, L) bytes.
 */
kvq_status kvq_fp16_qk_matvec(const uint16_t *d_k16, int64_t L, int32_t n_kv_heads, int32_t n_q_heads,
                              const float *d_q, float scale, float *d_scores, int64_t ld_scores,
                              void *stream);
int64_t kvq_fp16_pv_workspace_bytes(int32_t n_q_heads, int64_t L);
kvq_status kvq_fp16_pv_matvec(const uint16_t *d_v16, int64_t L, int32_t n_kv_heads, int32_t n_q_heads,
                              const float *d_probs, int64_t ld_probs, float *d_out,
                              void *d_workspace, int64_t workspace_bytes, void *stream);

/*
 * Streaming-read reference for the bandwidth figures (no part of the method): reads `bytes` bytes of
 * d_buf once with 16-byte loads and leaves per-workgroup checksums (sum over the workgroup's 16-byte
 * groups of the XOR of their four 32-bit words, as uint32) in d_workspace; the time of this call is
 * what a kernel that only reads can reach on this GPU.
 *   d_buf: DEVICE, 16-byte aligned, bytes a positive multiple of 16.
 *   d_workspace: DEVICE, kvq_stream_read_workspace_bytes() bytes.
 * Errors: INVALID_ARG, CAPACITY (workspace), HIP.
 */
int64_t kvq_stream_read_workspace_bytes(void);
kvq_status kvq_stream_read(const void *d_buf, int64_t bytes, void *d_workspace, int64_t workspace_bytes,
                           void *stream);

/*
 * Timing aid: runs `fn`-independent HIP events on `stream`.  kvq_event_* wrap hipEvent so that a
 * Python caller can time work on the stream the kernels are launched on without another binding.
 */
kvq_status kvq_event_create(void **event);
kvq_status kvq_event_record(void *event, void *stream);
kvq_status kvq_event_elapsed_ms(void *start, void *stop, float *ms); /* synchronizes on stop */
kvq_status kvq_event_destroy(void *event);

/*
 * Per-kernel timing aid for benchmarks, for the dense kernel of kvq_qk_matvec / kvq_pv_matvec /
 * kvq_attention_decode (`which`: 0 = QK dense kernel, 1 = PV dense kernel).  Two measurements, each
 * kept per call in a ring of 256, so that many calls can be timed back to back without waiting for
 * the GPU in between:
 *   events : a pair of HIP events recorded on the launch stream around the launch.  The interval runs
 *            from the end of the kernel before to the end of this one, and every record stalls the
 *            queue by a few microseconds: an upper bound on the kernel's duration.
 *   span   : every workgroup of the kernel stores the GPU's constant-rate wall clock when it starts
 *            and when its last wavefront's stores have been acknowledged, in a slot of its own in a
 *            caller-provided DEVICE buffer; first start to last end over the workgroups is the span a
 *            kernel trace reports for the launch, and nothing is inserted between kernels.  (Launches
 *            of more than 1024 workgroups are not timed this way, nor the Key kernel variants that
 *            keep eight query heads per thread: kvq_profile_span_us then returns INVALID_ARG.  The
 *            3-bit Key kernel for tiles of 1024 tokens keeps one shared pair of words instead of a
 *            slot per workgroup, earliest start and latest end by atomic minimum and maximum, and
 *            finds them through a pointer in device memory that a one-workgroup kernel sets ahead
 *            of the call's first launch while spans are being taken.)
 *   kvq_profile_set_span_buffer(d_buf, bytes): DEVICE buffer of kvq_profile_span_buffer_bytes()
 *     bytes, 8-byte aligned, owned by the caller and kept until spans are switched off again with a
 *     null pointer; only while the aid is disabled.
 *   kvq_profile_enable(on): 0 = off; 1 = events (and spans if a buffer is set); 3 = spans only, no
 *     event records.  Enabling resets the call counts and, with a buffer, synchronizes the device and
 *     clears the buffer.
 *   kvq_profile_count: calls recorded since then.
 *   kvq_profile_read_ms / kvq_profile_last_ms: event interval of call number `call` (0-based; one of
 *     the last 256) / of the most recent call; synchronizes on that call's stop event.
 *   kvq_profile_span_us: span of call number `call`; synchronizes the device.
 * Not thread-safe; leave disabled in production.  Errors: INVALID_ARG (which, call out of range,
 * measurement not being taken, buffer too small or set while enabled), HIP.
 */
kvq_status kvq_profile_enable(int32_t on);
int64_t kvq_profile_span_buffer_bytes(void);
kvq_status kvq_profile_set_span_buffer(void *d_buf, int64_t bytes);
kvq_status kvq_profile_count(int32_t which, int64_t *count);
kvq_status kvq_profile_read_ms(int32_t which, int64_t call, float *ms);
kvq_status kvq_profile_last_ms(int32_t which, float *ms);
kvq_status kvq_profile_span_us(int32_t which, int64_t call, float *us);

#ifdef __cplusplus
}
#endif
#endif /* KVQ_H */
