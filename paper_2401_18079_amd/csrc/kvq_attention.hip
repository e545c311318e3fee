// Fused decode-step attention: scores, softmax and output in one call (paper Sec. 3: generation-time
// attention is the two mat-vecs q.K^T and p.V with a softmax between them).  The softmax never runs
// as passes of its own: the Key kernels leave per-workgroup score maxima next to the scores, the
// Value kernels weight token n by exp(x_n - max) as they load its score and sum the weights on the
// way, and the final reduction divides by that sum.
#include <mutex>
#include "kvq_common.hpp"

// Scratch of kvq_attention_decode_noalloc: the slab partials of the Value kernels and the softmax
// statistics of the Key kernels, for up to KVQ_NOALLOC_MAX_Q_HEADS query heads.  One copy per GPU,
// held until the process ends.  In host code this name is only a handle for hipGetSymbolAddress: the
// address kernels may use is the one that call returns, per device.
static constexpr int KVQ_NOALLOC_MAX_DEVICES = 64;
static constexpr int64_t KVQ_NOALLOC_PV_BYTES =
    ((int64_t)512 * KVQ_NOALLOC_MAX_Q_HEADS * 128 * 2 + (int64_t)512 * KVQ_NOALLOC_MAX_Q_HEADS * 2) * 4;
static constexpr int64_t KVQ_NOALLOC_BYTES =
    KVQ_NOALLOC_PV_BYTES + (int64_t)KVQ_NOALLOC_MAX_Q_HEADS * KVQ_STAT_SLOTS * (int64_t)sizeof(float);
static __device__ __align__(256) unsigned char kvq_noalloc_scratch[KVQ_NOALLOC_BYTES];

// Device address of the scratch array on the current device (looked up once per device).
static kvq_status kvq_noalloc_scratch_ptr(void **out)
{
    static std::mutex mu;
    static void *ptrs[KVQ_NOALLOC_MAX_DEVICES] = {};
    int dev = 0;
    KVQ_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= KVQ_NOALLOC_MAX_DEVICES) return KVQ_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void *p = nullptr;
        KVQ_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(kvq_noalloc_scratch)));
        if (!p) return KVQ_ERR_HIP;
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return KVQ_OK;
}

extern "C" kvq_status kvq_attention_decode(const kvq_cache *cache, const float *d_q_rot, float scale, float *d_scores,
                                           int64_t ld_scores, float *d_out, void *stream)
{
    kvq_status st = kvq_check_cache(cache);
    if (st != KVQ_OK) return st;
    if (cache->n_tokens_k != cache->n_tokens_v) return KVQ_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const int64_t pv_bytes = kvq_pv_workspace_bytes(cache->n_q_heads);
    const int64_t stat_bytes = (int64_t)cache->n_q_heads * KVQ_STAT_SLOTS * (int64_t)sizeof(float);
    if (!cache->workspace || cache->workspace_bytes < pv_bytes + stat_bytes) return KVQ_ERR_CAPACITY;
    float *slots = (float *)((char *)cache->workspace + pv_bytes);
    int n_stat = 0;
    st = kvq_qk_run(cache, d_q_rot, scale, d_scores, ld_scores, slots, &n_stat, s);
    if (st != KVQ_OK) return st;
    // an empty cache has no statistics: the Value half then sums nothing and writes zeros
    return kvq_pv_run(cache, d_scores, ld_scores, d_out, n_stat > 0 ? slots : nullptr, n_stat, s);
}

extern "C" kvq_status kvq_attention_decode_noalloc(const kvq_cache *cache, const float *d_q_rot, float scale,
                                                   float *d_scores, int64_t ld_scores, float *d_out, void *stream)
{
    kvq_status st = kvq_check_cache(cache);
    if (st != KVQ_OK) return st;
    if (cache->n_q_heads > KVQ_NOALLOC_MAX_Q_HEADS) return KVQ_ERR_CAPACITY;
    static_assert(KVQ_NOALLOC_MAX_Q_HEADS == 32, "the header states the limit");
    if (kvq_pv_workspace_bytes(cache->n_q_heads) > KVQ_NOALLOC_PV_BYTES) return KVQ_ERR_CAPACITY;
    void *scratch = nullptr;
    st = kvq_noalloc_scratch_ptr(&scratch);
    if (st != KVQ_OK) return st;
    // the same kernels as kvq_attention_decode, on a copy of the descriptor whose workspace is the
    // static array (every slot that is read is written first by the kernels: nothing to clear)
    kvq_cache view = *cache;
    view.workspace = scratch;
    view.workspace_bytes = KVQ_NOALLOC_BYTES;
    return kvq_attention_decode(&view, d_q_rot, scale, d_scores, ld_scores, d_out, stream);
}

// One generation step in one call: append the new token's Key and Value, then attend over the cache
// that now ends with it.  Everything the host can check for the attention half is checked before
// the append is launched, so that a rejected call leaves the cache as it was.
extern "C" kvq_status kvq_decode_step(kvq_cache *cache, const uint16_t *d_k_new, const uint16_t *d_v_new,
                                      const float *d_q_rot, float scale, float *d_scores, int64_t ld_scores,
                                      float *d_out, void *stream)
{
    kvq_status st = kvq_check_cache(cache);
    if (st != KVQ_OK) return st;
    if (!cache->loaded) return KVQ_ERR_NOT_LOADED;
    if (cache->n_tokens_k != cache->n_tokens_v) return KVQ_ERR_INVALID_ARG;
    if (!d_q_rot || !d_scores || !d_out || ((uintptr_t)d_q_rot & 3) || ((uintptr_t)d_scores & 3) ||
        ((uintptr_t)d_out & 3))
        return KVQ_ERR_INVALID_ARG;
    if (ld_scores < cache->n_tokens_k + 1) return KVQ_ERR_INVALID_ARG;
    const int64_t need = kvq_pv_workspace_bytes(cache->n_q_heads) +
                         (int64_t)cache->n_q_heads * KVQ_STAT_SLOTS * (int64_t)sizeof(float);
    if (!cache->workspace || cache->workspace_bytes < need) return KVQ_ERR_CAPACITY;
    // the append and the sparse Key kernel over the tokens before it as one launch, where that is built
    bool front = false;
    st = kvq_step_front_launch(cache, d_k_new, d_v_new, d_q_rot, scale, d_scores, ld_scores, (hipStream_t)stream, &front);
    if (st != KVQ_OK) return st;
    if (front) {
        kvq_cache view = *cache;
        view.loaded |= KVQ_LOADED_SPARSE_SCORES_DONE;
        return kvq_attention_decode(&view, d_q_rot, scale, d_scores, ld_scores, d_out, stream);
    }
    st = kvq_quantize_append_kv(cache, d_k_new, d_v_new, 1, stream);
    if (st != KVQ_OK) return st;
    return kvq_attention_decode(cache, d_q_rot, scale, d_scores, ld_scores, d_out, stream);
}
