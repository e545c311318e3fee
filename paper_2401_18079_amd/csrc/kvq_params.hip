// Host-side helpers of the C ABI and kvq_lut_load (stages one layer's quantization constants).
#include <math.h>
#include <string.h>
#include "kvq_common.hpp"

extern "C" {

int64_t kvq_codes_bytes(int32_t bits, int32_t n_kv_heads, int64_t cap_tokens)
{
    return (int64_t)n_kv_heads * cap_tokens * 16 * bits;
}

int64_t kvq_params_bytes(int32_t n_kv_heads)
{
    int64_t b = kvq_params_bytes_D(n_kv_heads * KVQ_HEAD_DIM);
    return (b + 255) & ~(int64_t)255;
}

const char *kvq_status_string(kvq_status s)
{
    switch (s) {
    case KVQ_OK: return "ok";
    case KVQ_ERR_INVALID_ARG: return "invalid argument";
    case KVQ_ERR_UNSUPPORTED: return "unsupported shape or bit width";
    case KVQ_ERR_CAPACITY: return "capacity exceeded";
    case KVQ_ERR_NNZ_OVERFLOW: return "sparse outlier array full";
    case KVQ_ERR_NOT_LOADED: return "kvq_lut_load not called";
    case KVQ_ERR_HIP: return "HIP runtime error";
    }
    return "unknown";
}

const char *kvq_version(void) { return "kvq 0.2 (gfx950)"; }

static float kvq_signpost_fp16(float x);
float kvq_stored_signpost(float x) { return (fabsf(x) < 65520.0f) ? kvq_signpost_fp16(x) : NAN; }

kvq_status kvq_event_create(void **event)
{
    if (!event) return KVQ_ERR_INVALID_ARG;
    hipEvent_t e;
    KVQ_HIP_CHECK(hipEventCreate(&e));
    *event = (void *)e;
    return KVQ_OK;
}
kvq_status kvq_event_record(void *event, void *stream)
{
    KVQ_HIP_CHECK(hipEventRecord((hipEvent_t)event, (hipStream_t)stream));
    return KVQ_OK;
}
kvq_status kvq_event_elapsed_ms(void *start, void *stop, float *ms)
{
    if (!ms) return KVQ_ERR_INVALID_ARG;
    KVQ_HIP_CHECK(hipEventSynchronize((hipEvent_t)stop));
    KVQ_HIP_CHECK(hipEventElapsedTime(ms, (hipEvent_t)start, (hipEvent_t)stop));
    return KVQ_OK;
}
kvq_status kvq_event_destroy(void *event)
{
    KVQ_HIP_CHECK(hipEventDestroy((hipEvent_t)event));
    return KVQ_OK;
}

kvq_status kvq_profile_enable(int32_t on)
{
    KvqProfile &p = kvq_profile_state();
    if (on && !p.ev[0][0][0]) {
        for (int k = 0; k < 2; ++k)
            for (int i = 0; i < KVQ_PROFILE_RING; ++i)
                for (int j = 0; j < 2; ++j)
                    // no system-scope fence at the record: the bracket should disturb the kernels as little as possible
                    KVQ_HIP_CHECK(hipEventCreateWithFlags(&p.ev[k][i][j], hipEventDisableSystemFence));
    }
    if (on) {
        p.count[0] = p.count[1] = 0;
        p.use_events = (on & 2) ? 0 : 1;                 // bit 1: spans only, nothing recorded between kernels
        if (p.spans) {
            KVQ_HIP_CHECK(hipDeviceSynchronize());
            KVQ_HIP_CHECK(hipMemset(p.spans, 0, (size_t)kvq_profile_span_buffer_bytes()));
        }
    }
    p.enabled = on ? 1 : 0;
    return KVQ_OK;
}

int64_t kvq_profile_span_buffer_bytes(void) { return (int64_t)2 * KVQ_PROFILE_RING * KVQ_PROFILE_MAX_WGS * 2 * 8; }

kvq_status kvq_profile_set_span_buffer(void *d_buf, int64_t bytes)
{
    KvqProfile &p = kvq_profile_state();
    if (p.enabled) return KVQ_ERR_INVALID_ARG;
    if (d_buf && (((uintptr_t)d_buf & 7) || bytes < kvq_profile_span_buffer_bytes())) return KVQ_ERR_INVALID_ARG;
    p.spans = (unsigned long long *)d_buf;
    return KVQ_OK;
}

kvq_status kvq_profile_span_us(int32_t which, int64_t call, float *us)
{
    KvqProfile &p = kvq_profile_state();
    if (which < 0 || which > 1 || !us || !p.spans) return KVQ_ERR_INVALID_ARG;
    if (call < 0 || call >= p.count[which] || call + KVQ_PROFILE_RING < p.count[which]) return KVQ_ERR_INVALID_ARG;
    static unsigned long long host[KVQ_PROFILE_MAX_WGS * 2];
    const unsigned long long *slots =
        p.spans + ((int64_t)which * KVQ_PROFILE_RING + (call % KVQ_PROFILE_RING)) * KVQ_PROFILE_MAX_WGS * 2;
    KVQ_HIP_CHECK(hipDeviceSynchronize());
    KVQ_HIP_CHECK(hipMemcpy(host, slots, sizeof(host), hipMemcpyDeviceToHost));
    int dev = 0, khz = 0;
    KVQ_HIP_CHECK(hipGetDevice(&dev));
    KVQ_HIP_CHECK(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    if (khz <= 0) return KVQ_ERR_HIP;
    // first start to last end over the workgroups that ran (an unused slot is zero)
    unsigned long long first = ~0ull, last = 0;
    for (int w = 0; w < KVQ_PROFILE_MAX_WGS; ++w) {
        if (host[2 * w] == 0 || host[2 * w + 1] == 0) continue;
        if (host[2 * w] < first) first = host[2 * w];
        if (host[2 * w + 1] > last) last = host[2 * w + 1];
    }
    if (last < first) return KVQ_ERR_INVALID_ARG;        // the launch was too large for its slots, or did not run
    const unsigned long long best = last - first;
    *us = (float)((double)best * 1000.0 / (double)khz);
    return KVQ_OK;
}

kvq_status kvq_profile_count(int32_t which, int64_t *count)
{
    KvqProfile &p = kvq_profile_state();
    if (which < 0 || which > 1 || !count) return KVQ_ERR_INVALID_ARG;
    *count = p.count[which];
    return KVQ_OK;
}

kvq_status kvq_profile_read_ms(int32_t which, int64_t call, float *ms)
{
    KvqProfile &p = kvq_profile_state();
    if (which < 0 || which > 1 || !ms || !p.use_events) return KVQ_ERR_INVALID_ARG;
    if (call < 0 || call >= p.count[which] || call + KVQ_PROFILE_RING < p.count[which]) return KVQ_ERR_INVALID_ARG;
    hipEvent_t *e = p.ev[which][call % KVQ_PROFILE_RING];
    KVQ_HIP_CHECK(hipEventSynchronize(e[1]));
    KVQ_HIP_CHECK(hipEventElapsedTime(ms, e[0], e[1]));
    return KVQ_OK;
}

kvq_status kvq_profile_last_ms(int32_t which, float *ms)
{
    KvqProfile &p = kvq_profile_state();
    if (which < 0 || which > 1) return KVQ_ERR_INVALID_ARG;
    return kvq_profile_read_ms(which, p.count[which] - 1, ms);
}

}  // extern "C"

KvqProfile &kvq_profile_state()
{
    static KvqProfile p = {};
    return p;
}

// A signpost as the library stores it: the fp32 value of the nearest fp16 number (ties to even).  The
// paper's look-up tables hold fp16 entries (App. "Kernel Implementation Details"), and with signposts
// that are fp16 numbers the fp16 pair table of the dense Value kernel is exact, so append, scores and
// outputs all see one and the same table.  Signposts lie in [-1, 1]: the mantissa is rounded in the
// fp32 bit pattern (normal range of fp16) or on the 2^-24 grid (below 2^-14).  |x| < 65520 (checked
// by the caller: beyond that fp16 has no finite neighbour).
static float kvq_signpost_fp16(float x)
{
    if (fabsf(x) < 6.103515625e-05f) {                       // subnormal range of fp16: multiples of 2^-24
        const float q = nearbyintf(x * 16777216.0f);         // exact product, ties to even
        return q * (1.0f / 16777216.0f);
    }
    uint32_t b;
    memcpy(&b, &x, 4);
    const uint32_t keep = b & ~0x1FFFu, rest = b & 0x1FFFu;  // 13 mantissa bits go
    uint32_t r = keep;
    if (rest > 0x1000u || (rest == 0x1000u && (keep & 0x2000u))) r += 0x2000u;   // may carry into the exponent
    float y;
    memcpy(&y, &r, 4);
    return y;
}

// Expand the fp16 per-channel constants to fp32 and form the reciprocal scale with one IEEE division,
// so every later kernel normalises with exactly (x - z) * (1/s).
__global__ void kvq_params_expand(void *block, int D)
{
    KvqParamsView v = kvq_params_view(block, D);
    int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= D) return;
    float s = kvq_h2f(v.s16[c]);
    ((float *)v.s)[c] = s;
    ((float *)v.z)[c] = kvq_h2f(v.z16[c]);
    ((float *)v.rinv)[c] = __fdiv_rn(1.0f, s);
    ((float *)v.lo)[c] = kvq_h2f(v.lo16[c]);
    ((float *)v.hi)[c] = kvq_h2f(v.hi16[c]);
}

extern "C" kvq_status kvq_lut_load(kvq_cache *cache, const float *h_lut_k, const float *h_lut_v,
                                   const uint16_t *h_s_k, const uint16_t *h_z_k,
                                   const uint16_t *h_lo_k, const uint16_t *h_hi_k, void *stream)
{
    kvq_status st = kvq_check_cache(cache);
    if (st != KVQ_OK) return st;
    if (!h_lut_k || !h_lut_v || !h_s_k || !h_z_k || !h_lo_k || !h_hi_k) return KVQ_ERR_INVALID_ARG;
    if (!(cache->rope_base > 1.0f)) return KVQ_ERR_INVALID_ARG;
    const int D = cache->n_kv_heads * KVQ_HEAD_DIM;
    const int ne = 1 << cache->bits;
    for (int j = 1; j < ne; ++j)
        if (!(h_lut_k[j] >= h_lut_k[j - 1]) || !(h_lut_v[j] >= h_lut_v[j - 1])) return KVQ_ERR_INVALID_ARG;
    for (int j = 0; j < ne; ++j)        // finite and within the range of fp16 (also rejects NaN)
        if (!(fabsf(h_lut_k[j]) < 65520.0f) || !(fabsf(h_lut_v[j]) < 65520.0f)) return KVQ_ERR_INVALID_ARG;

    KvqParamsHeader hdr;
    memset(&hdr, 0, sizeof(hdr));
    for (int j = 0; j < ne; ++j) { hdr.lut_k[j] = kvq_signpost_fp16(h_lut_k[j]); hdr.lut_v[j] = kvq_signpost_fp16(h_lut_v[j]); }
    for (int i = 0; i < 64; ++i) {
        // rotation frequency of channel pair (i, i+64) in revolutions per position, split in two floats
        double rev = pow((double)cache->rope_base, -2.0 * (double)i / (double)KVQ_HEAD_DIM) / (2.0 * M_PI);
        float hi = (float)rev;
        hdr.rope_vh[i] = hi;
        hdr.rope_vl[i] = (float)(rev - (double)hi);
        // rotation by KVQ_ROPE_STEP positions: the angle is reduced in double before cos / sin
        const double step = fmod((double)KVQ_ROPE_STEP * rev, 1.0) * (2.0 * M_PI);
        hdr.rope_cd[i] = (float)cos(step);
        hdr.rope_sd[i] = (float)sin(step);
    }
    hdr.D = D;
    hdr.bits = cache->bits;
    hipStream_t s = (hipStream_t)stream;
    KVQ_HIP_CHECK(hipStreamSynchronize(s));
    char *blk = (char *)cache->params;
    KVQ_HIP_CHECK(hipMemcpy(blk, &hdr, sizeof(hdr), hipMemcpyHostToDevice));
    KVQ_HIP_CHECK(hipMemcpy(blk + KVQ_PARAMS_HEADER_BYTES, h_s_k, 2 * (size_t)D, hipMemcpyHostToDevice));
    KVQ_HIP_CHECK(hipMemcpy(blk + KVQ_PARAMS_HEADER_BYTES + 2 * (size_t)D, h_z_k, 2 * (size_t)D, hipMemcpyHostToDevice));
    KVQ_HIP_CHECK(hipMemcpy(blk + KVQ_PARAMS_HEADER_BYTES + 4 * (size_t)D, h_lo_k, 2 * (size_t)D, hipMemcpyHostToDevice));
    KVQ_HIP_CHECK(hipMemcpy(blk + KVQ_PARAMS_HEADER_BYTES + 6 * (size_t)D, h_hi_k, 2 * (size_t)D, hipMemcpyHostToDevice));
    kvq_params_expand<<<(D + 255) / 256, 256, 0, s>>>(cache->params, D);
    KVQ_HIP_CHECK(hipGetLastError());
    // bit 0: loaded; bit 1: the thresholds admit no Key outlier at all (every finite fp16 passes), so
    // the score kernel can skip the sparse part
    bool no_outliers = true;
    for (int c = 0; c < D && no_outliers; ++c)
        no_outliers = (h_lo_k[c] == 0xFBFFu) && (h_hi_k[c] == 0x7BFFu);   // -65504 / +65504
    cache->loaded = no_outliers ? 3 : 1;
    return KVQ_OK;
}
