// Row-wise fp32 softmax with max subtraction (helper between the two mat-vecs of a decode step).
// Two passes: per-chunk (max, sum of exp) pairs, then every chunk combines all pairs of its row and
// normalises its own slice.  Rows are long (the context), so each row is split over many workgroups.
#include "kvq_common.hpp"

namespace {

constexpr int SM_NT = 256;
constexpr int SM_CHUNK = 4096;     // elements per workgroup

__device__ inline void block_max_sum(float &m, float &s, float *sh_m, float *sh_s)
{
    // combine (m, s) pairs of all threads: s is a sum of exp(x - m)
    for (int o = 32; o > 0; o >>= 1) {
        float m2 = __shfl_xor(m, o), s2 = __shfl_xor(s, o);
        float mn = fmaxf(m, m2);
        s = s * __expf(m - mn) + s2 * __expf(m2 - mn);
        m = mn;
    }
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { sh_m[w] = m; sh_s[w] = s; }
    __syncthreads();
    m = sh_m[0]; s = sh_s[0];
    for (int i = 1; i < SM_NT / 64; ++i) {
        float mn = fmaxf(m, sh_m[i]);
        s = s * __expf(m - mn) + sh_s[i] * __expf(sh_m[i] - mn);
        m = mn;
    }
    __syncthreads();
}

// The SM_CHUNK elements a workgroup owns, SM_CHUNK / SM_NT per thread, read once into registers.
// VEC: rows are 16-byte aligned, so a thread takes groups of four consecutive elements with one
// 16-byte load each; otherwise element by element.  Elements past `n` read as `pad`.
template <bool VEC>
__device__ __forceinline__ void load_chunk(const float *__restrict__ xr, int64_t b, int64_t n, float pad,
                                           float (&v)[SM_CHUNK / SM_NT])
{
    constexpr int PER = SM_CHUNK / SM_NT;
    if (VEC) {
#pragma unroll
        for (int k = 0; k < PER / 4; ++k) {
            const int64_t i = b + ((int64_t)k * SM_NT + threadIdx.x) * 4;
            if (i + 3 < n) {
                const float4 q = *(const float4 *)(xr + i);
                v[4 * k + 0] = q.x; v[4 * k + 1] = q.y; v[4 * k + 2] = q.z; v[4 * k + 3] = q.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) v[4 * k + j] = (i + j < n) ? xr[i + j] : pad;
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int64_t i = b + threadIdx.x + (int64_t)k * SM_NT;
            v[k] = (i < n) ? xr[i] : pad;
        }
    }
}

// index of register element k of load_chunk
template <bool VEC>
__device__ __forceinline__ int64_t chunk_index(int64_t b, int k)
{
    return VEC ? b + ((int64_t)(k / 4) * SM_NT + threadIdx.x) * 4 + (k & 3) : b + threadIdx.x + (int64_t)k * SM_NT;
}

template <bool VEC>
__global__ __launch_bounds__(SM_NT) void kvq_softmax_partial(const float *__restrict__ x, int64_t ld, int64_t n,
                                                             float2_t *__restrict__ ws, int chunks)
{
    __shared__ float sh_m[SM_NT / 64], sh_s[SM_NT / 64];
    const int row = blockIdx.y, chunk = blockIdx.x;
    const float *xr = x + (int64_t)row * ld;
    const int64_t b = (int64_t)chunk * SM_CHUNK;
    constexpr int PER = SM_CHUNK / SM_NT;          // elements per thread, read once and kept in registers
    float v[PER];
    load_chunk<VEC>(xr, b, n, -INFINITY, v);
    float m = -INFINITY;
#pragma unroll
    for (int k = 0; k < PER; ++k) m = fmaxf(m, v[k]);
    float s = 0.f;
    // threads without elements: a finite floor instead of -inf keeps exp(m - m') free of inf - inf
    if (m == -INFINITY) m = -3.0e38f;
#pragma unroll
    for (int k = 0; k < PER; ++k) s += __expf(v[k] - m);        // exp(-inf) = 0 for the padding
    block_max_sum(m, s, sh_m, sh_s);
    if (threadIdx.x == 0) ws[(int64_t)row * chunks + chunk] = float2_t{m, s};
}

template <bool VEC>
__global__ __launch_bounds__(SM_NT) void kvq_softmax_finish(const float *__restrict__ x, int64_t ld_x,
                                                            float *__restrict__ y, int64_t ld_y, int64_t n,
                                                            const float2_t *__restrict__ ws, int chunks)
{
    __shared__ float sh_m[SM_NT / 64], sh_s[SM_NT / 64];
    const int row = blockIdx.y, chunk = blockIdx.x;
    float m = -INFINITY, s = 0.f;
    for (int c = threadIdx.x; c < chunks; c += SM_NT) {
        const float2_t v = ws[(int64_t)row * chunks + c];
        float mn = fmaxf(m, v.x);
        if (mn != -INFINITY) s = s * __expf(m - mn) + v.y * __expf(v.x - mn);
        m = mn;
    }
    if (m == -INFINITY) { s = 0.f; }
    // -inf - -inf would be NaN inside the combine: give idle threads a finite floor
    if (m == -INFINITY) m = -3.0e38f;
    block_max_sum(m, s, sh_m, sh_s);
    const float inv = 1.0f / s;
    const float *xr = x + (int64_t)row * ld_x;
    float *yr = y + (int64_t)row * ld_y;
    const int64_t b = (int64_t)chunk * SM_CHUNK;
    constexpr int PER = SM_CHUNK / SM_NT;
    float v[PER];
    load_chunk<VEC>(xr, b, n, 0.f, v);
    if (VEC) {
#pragma unroll
        for (int k = 0; k < PER / 4; ++k) {
            const int64_t i = chunk_index<VEC>(b, 4 * k);
            float4 q;
            q.x = __expf(v[4 * k + 0] - m) * inv; q.y = __expf(v[4 * k + 1] - m) * inv;
            q.z = __expf(v[4 * k + 2] - m) * inv; q.w = __expf(v[4 * k + 3] - m) * inv;
            if (i + 3 < n) {
                *(float4 *)(yr + i) = q;
            } else {
                const float e[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (i + j < n) yr[i + j] = e[j];
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int64_t i = chunk_index<VEC>(b, k);
            if (i < n) yr[i] = __expf(v[k] - m) * inv;
        }
    }
}

}  // namespace

extern "C" int64_t kvq_softmax_workspace_bytes(int32_t n_rows, int64_t n_cols)
{
    int64_t chunks = (n_cols + SM_CHUNK - 1) / SM_CHUNK;
    if (chunks < 1) chunks = 1;
    return (((int64_t)n_rows * chunks * 8) + 255) & ~(int64_t)255;
}

extern "C" kvq_status kvq_softmax_f32(const float *d_x, int64_t ld_x, float *d_probs, int64_t ld_probs,
                                      int32_t n_rows, int64_t n_cols, void *d_workspace, int64_t workspace_bytes,
                                      void *stream)
{
    if (!d_x || !d_probs || n_rows < 1 || n_cols < 1 || ld_x < n_cols || ld_probs < n_cols) return KVQ_ERR_INVALID_ARG;
    if (!d_workspace || workspace_bytes < kvq_softmax_workspace_bytes(n_rows, n_cols)) return KVQ_ERR_CAPACITY;
    const int chunks = (int)((n_cols + SM_CHUNK - 1) / SM_CHUNK);
    hipStream_t s = (hipStream_t)stream;
    dim3 grid((unsigned)chunks, (unsigned)n_rows);
    // 16-byte loads and stores when every row of both matrices starts on a 16-byte boundary
    const bool vec = !(((uintptr_t)d_x | (uintptr_t)d_probs) & 15) && !((ld_x | ld_probs) & 3);
    if (vec) {
        kvq_softmax_partial<true><<<grid, SM_NT, 0, s>>>(d_x, ld_x, n_cols, (float2_t *)d_workspace, chunks);
        kvq_softmax_finish<true><<<grid, SM_NT, 0, s>>>(d_x, ld_x, d_probs, ld_probs, n_cols,
                                                        (const float2_t *)d_workspace, chunks);
    } else {
        kvq_softmax_partial<false><<<grid, SM_NT, 0, s>>>(d_x, ld_x, n_cols, (float2_t *)d_workspace, chunks);
        kvq_softmax_finish<false><<<grid, SM_NT, 0, s>>>(d_x, ld_x, d_probs, ld_probs, n_cols,
                                                         (const float2_t *)d_workspace, chunks);
    }
    KVQ_HIP_CHECK(hipGetLastError());
    return KVQ_OK;
}
