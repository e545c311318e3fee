// Same-GPU fp16-cache baselines: plain mat-vecs against an uncompressed fp16 Key cache (already
// rotated) and Value cache, in the same output layout as the quantized path.  These are what the
// quantized kernels are compared with (the paper compares against fp16 mat-vec kernels, Sec. 4.4).
#include "kvq_common.hpp"

namespace {

// scores[q][n] = scale * sum_c q[q][c] * K16[n][kv(q)*128+c].
// 16 lanes cover one (token, KV head) row of 128 fp16 (8 each); a wavefront covers 4 KV heads of
// one token per step; each lane keeps its 8 query values per query head of the group in registers.
template <int R>
__global__ __launch_bounds__(256) void fp16_qk(const uint16_t *__restrict__ k16, int64_t L, int n_kv_heads,
                                               const float *__restrict__ q, float scale,
                                               float *__restrict__ scores, int64_t ld, int tokens_per_wg)
{
    const int D = n_kv_heads * 128;
    const int lanes_per_row = D / 8;                      // 16-byte vectors per token row
    const int tid = threadIdx.x;
    const int sub = tid & 15;                             // which 8 channels of the head
    // thread handles vector index v = vbase + k*256 of each token row
    for (int v = tid; v < lanes_per_row; v += 256) {
        const int kvh = v >> 4;
        float qv[R][8];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int j = 0; j < 8; ++j) qv[r][j] = q[(kvh * R + r) * 128 + sub * 8 + j] * scale;
        const int64_t n0 = (int64_t)blockIdx.x * tokens_per_wg;
        for (int t = 0; t < tokens_per_wg; ++t) {
            const int64_t n = n0 + t;
            if (n >= L) break;
            const uint4 raw = kvq_load_stream16(k16 + n * D + (int64_t)v * 8);
            const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
            float acc[R];
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r] = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const half2_t h = __builtin_bit_cast(half2_t, w[j]);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    acc[r] = __builtin_fmaf((float)h.x, qv[r][2 * j], acc[r]);
                    acc[r] = __builtin_fmaf((float)h.y, qv[r][2 * j + 1], acc[r]);
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                float a = acc[r];
                a += __shfl_xor(a, 1); a += __shfl_xor(a, 2); a += __shfl_xor(a, 4); a += __shfl_xor(a, 8);
                if (sub == 0) scores[(int64_t)(kvh * R + r) * ld + n] = a;
            }
        }
    }
}

// partial[slab][q][c] = sum_{n in slab} p[q][n] * V16[n][kv(q)*128+c]
template <int R>
__global__ __launch_bounds__(256) void fp16_pv(const uint16_t *__restrict__ v16, int64_t L, int n_kv_heads,
                                               const float *__restrict__ probs, int64_t ld,
                                               float *__restrict__ partial, int64_t tokens_per_slab)
{
    const int D = n_kv_heads * 128, n_q_heads = n_kv_heads * R;
    const int lanes_per_row = D / 8;
    const int tid = threadIdx.x;
    const int64_t nb = (int64_t)blockIdx.x * tokens_per_slab;
    int64_t ne = nb + tokens_per_slab;
    if (ne > L) ne = L;
    for (int v = tid; v < lanes_per_row; v += 256) {
        const int kvh = v >> 4, sub = v & 15;
        float acc[R][8];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[r][j] = 0.f;
        constexpr int U = 8;                       // token rows in flight per thread
        for (int64_t n0 = nb; n0 < ne; n0 += U) {
            uint4 raw[U];
            float pr[U][R];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t n = (n0 + u < ne) ? n0 + u : ne - 1;   // clamped: straight-line loads
                raw[u] = kvq_load_stream16(v16 + n * D + (int64_t)v * 8);
#pragma unroll
                for (int r = 0; r < R; ++r)
                    pr[u][r] = (n0 + u < ne) ? probs[(int64_t)(kvh * R + r) * ld + n] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t w[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
#pragma unroll
                for (int r = 0; r < R; ++r) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const half2_t h = __builtin_bit_cast(half2_t, w[j]);
                        acc[r][2 * j] = __builtin_fmaf((float)h.x, pr[u][r], acc[r][2 * j]);
                        acc[r][2 * j + 1] = __builtin_fmaf((float)h.y, pr[u][r], acc[r][2 * j + 1]);
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                partial[((int64_t)blockIdx.x * n_q_heads + kvh * R + r) * 128 + sub * 8 + j] = acc[r][j];
    }
}

__global__ __launch_bounds__(1024) void fp16_pv_reduce(int n_q_heads, int slabs, const float *__restrict__ partial,
                                                       float *__restrict__ out)
{
    __shared__ float red[8][128];
    const int qh = blockIdx.x, c = threadIdx.x & 127, j = threadIdx.x >> 7;
    float s = 0.f;
    for (int k0 = j; k0 < slabs; k0 += 64) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + 8 * u;
            v[u] = (k < slabs) ? partial[((int64_t)k * n_q_heads + qh) * 128 + c] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    red[j][c] = s;
    __syncthreads();
    if (j == 0) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) t += red[i][c];
        out[qh * 128 + c] = t;
    }
}

constexpr int FP16_PV_SLABS = 1024;

// Plain streaming read: every workgroup walks its share of the buffer in 16-byte loads (eight in
// flight per lane) and leaves one partial sum, so nothing but the reads limits it.  The loads carry
// the non-temporal hint; measured over 4 GiB: 6.4 TB/s with it, 5.9 TB/s without, and 8192 workgroups
// of 256 threads striding through the buffer together beat both fewer workgroups and one contiguous
// chunk per workgroup.
constexpr int STREAM_NT = 256, STREAM_WGS = 8192, STREAM_UNROLL = 8;
__device__ __forceinline__ uint32_t stream_fold(const uint4 *p)
{
    const uint4 v = kvq_load_stream16(p);
    return v.x ^ v.y ^ v.z ^ v.w;
}
__global__ __launch_bounds__(STREAM_NT) void stream_read(const uint4 *__restrict__ buf, int64_t n16,
                                                          uint32_t *__restrict__ sums)
{
    uint32_t acc = 0;
    const int64_t stride = (int64_t)gridDim.x * STREAM_NT;
    int64_t i = (int64_t)blockIdx.x * STREAM_NT + threadIdx.x;
    for (; i + (STREAM_UNROLL - 1) * stride < n16; i += STREAM_UNROLL * stride) {
        uint32_t v[STREAM_UNROLL];
#pragma unroll
        for (int u = 0; u < STREAM_UNROLL; ++u) v[u] = stream_fold(buf + i + u * stride);
#pragma unroll
        for (int u = 0; u < STREAM_UNROLL; ++u) acc += v[u];
    }
    for (; i < n16; i += stride) acc += stream_fold(buf + i);
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    __shared__ uint32_t red[STREAM_NT / 64];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int w = 0; w < STREAM_NT / 64; ++w) t += red[w];
        sums[blockIdx.x] = t;
    }
}

}  // namespace

extern "C" int64_t kvq_stream_read_workspace_bytes(void) { return (int64_t)STREAM_WGS * 4; }

extern "C" kvq_status kvq_stream_read(const void *d_buf, int64_t bytes, void *d_workspace, int64_t workspace_bytes,
                                      void *stream)
{
    if (!d_buf || ((uintptr_t)d_buf & 15) || bytes < 16 || (bytes & 15)) return KVQ_ERR_INVALID_ARG;
    if (!d_workspace || workspace_bytes < kvq_stream_read_workspace_bytes()) return KVQ_ERR_CAPACITY;
    const int64_t n16 = bytes / 16;
    int64_t wgs = (n16 + STREAM_NT - 1) / STREAM_NT;
    if (wgs > STREAM_WGS) wgs = STREAM_WGS;
    stream_read<<<(unsigned)wgs, STREAM_NT, 0, (hipStream_t)stream>>>((const uint4 *)d_buf, n16, (uint32_t *)d_workspace);
    KVQ_HIP_CHECK(hipGetLastError());
    return KVQ_OK;
}

extern "C" kvq_status kvq_fp16_qk_matvec(const uint16_t *d_k16, int64_t L, int32_t n_kv_heads, int32_t n_q_heads,
                                         const float *d_q, float scale, float *d_scores, int64_t ld_scores,
                                         void *stream)
{
    if (!d_k16 || !d_q || !d_scores || L < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || ld_scores < L ||
        ((uintptr_t)d_k16 & 15))
        return KVQ_ERR_INVALID_ARG;
    const int tokens_per_wg = 32;
    const unsigned grid = (unsigned)((L + tokens_per_wg - 1) / tokens_per_wg);
    hipStream_t s = (hipStream_t)stream;
    switch (n_q_heads / n_kv_heads) {
    case 1: fp16_qk<1><<<grid, 256, 0, s>>>(d_k16, L, n_kv_heads, d_q, scale, d_scores, ld_scores, tokens_per_wg); break;
    case 2: fp16_qk<2><<<grid, 256, 0, s>>>(d_k16, L, n_kv_heads, d_q, scale, d_scores, ld_scores, tokens_per_wg); break;
    case 4: fp16_qk<4><<<grid, 256, 0, s>>>(d_k16, L, n_kv_heads, d_q, scale, d_scores, ld_scores, tokens_per_wg); break;
    default: return KVQ_ERR_UNSUPPORTED;
    }
    KVQ_HIP_CHECK(hipGetLastError());
    return KVQ_OK;
}

extern "C" int64_t kvq_fp16_pv_workspace_bytes(int32_t n_q_heads, int64_t L)
{
    (void)L;
    return (int64_t)FP16_PV_SLABS * n_q_heads * 128 * 4;
}

extern "C" kvq_status kvq_fp16_pv_matvec(const uint16_t *d_v16, int64_t L, int32_t n_kv_heads, int32_t n_q_heads,
                                         const float *d_probs, int64_t ld_probs, float *d_out, void *d_workspace,
                                         int64_t workspace_bytes, void *stream)
{
    if (!d_v16 || !d_probs || !d_out || L < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || ld_probs < L ||
        ((uintptr_t)d_v16 & 15))
        return KVQ_ERR_INVALID_ARG;
    if (!d_workspace || workspace_bytes < kvq_fp16_pv_workspace_bytes(n_q_heads, L)) return KVQ_ERR_CAPACITY;
    int64_t tps = (L + FP16_PV_SLABS - 1) / FP16_PV_SLABS;
    if (tps < 16) tps = 16;
    const int slabs = (int)((L + tps - 1) / tps);
    hipStream_t s = (hipStream_t)stream;
    float *partial = (float *)d_workspace;
    switch (n_q_heads / n_kv_heads) {
    case 1: fp16_pv<1><<<slabs, 256, 0, s>>>(d_v16, L, n_kv_heads, d_probs, ld_probs, partial, tps); break;
    case 2: fp16_pv<2><<<slabs, 256, 0, s>>>(d_v16, L, n_kv_heads, d_probs, ld_probs, partial, tps); break;
    case 4: fp16_pv<4><<<slabs, 256, 0, s>>>(d_v16, L, n_kv_heads, d_probs, ld_probs, partial, tps); break;
    default: return KVQ_ERR_UNSUPPORTED;
    }
    fp16_pv_reduce<<<n_q_heads, 1024, 0, s>>>(n_q_heads, slabs, partial, d_out);
    KVQ_HIP_CHECK(hipGetLastError());
    return KVQ_OK;
}
