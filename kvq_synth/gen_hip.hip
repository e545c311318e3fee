// On-device twin of kvq_synth/gen.py: the same counter-based synthetic Key / Value activations,
// bit for bit (integer hashing plus single correctly rounded fp32 operations), so multi-gigabyte
// caches can be filled without generating them on the host.  Input generation only: nothing of the
// quantization method lives here.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ inline uint64_t splitmix64(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ inline float spiked_normalish(uint64_t h)
{
    const int s = (int)(h & 0xFFFF) + (int)((h >> 16) & 0xFFFF) + (int)((h >> 32) & 0xFFFF) + (int)((h >> 48) & 0xFFFF);
    const float g = __fmul_rn((float)(s - 131070), (float)(1.0 / 37837.227));
    const float spike = ((splitmix64(h) & 127ull) == 0ull) ? 6.0f : 1.0f;
    return __fmul_rn(g, spike);
}

// out[t][c] = fp16( (g * row_scale[t]) * a[c] + mu[c] );  row_scale == nullptr means 1 (Keys).
__global__ void synth_fill(uint64_t key, int64_t t0, int64_t T, int D, const float *__restrict__ a,
                           const float *__restrict__ mu, const float *__restrict__ row_scale,
                           _Float16 *__restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T * D) return;
    const int64_t t = i / D;
    const int c = (int)(i - t * D);
    const uint64_t h = splitmix64(key ^ ((uint64_t)(t0 + t) << 16) ^ (uint64_t)c);
    float g = spiked_normalish(h);
    if (row_scale) g = __fmul_rn(g, row_scale[t]);
    const float x = __fadd_rn(__fmul_rn(g, a[c]), mu[c]);
    out[i] = (_Float16)x;
}

}  // namespace

extern "C" int kvq_synth_fill(uint64_t key, int64_t t0, int64_t T, int D, const float *d_a, const float *d_mu,
                              const float *d_row_scale, void *d_out, void *stream)
{
    if (T < 1 || D < 1 || !d_a || !d_mu || !d_out) return 1;
    const int64_t n = T * D;
    synth_fill<<<(unsigned)((n + 255) / 256), 256, 0, (hipStream_t)stream>>>(key, t0, T, D, d_a, d_mu, d_row_scale,
                                                                           (_Float16 *)d_out);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
