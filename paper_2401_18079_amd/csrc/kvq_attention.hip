// Fused decode-step attention: scores, softmax and output in one call (paper Sec. 3: generation-time
// attention is the two mat-vecs q.K^T and p.V with a softmax between them).  The softmax never runs
// as passes of its own: the Key kernels leave per-workgroup score maxima next to the scores, the
// Value kernels weight token n by exp(x_n - max) as they load its score and sum the weights on the
// way, and the final reduction divides by that sum.
#include "kvq_common.hpp"

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
