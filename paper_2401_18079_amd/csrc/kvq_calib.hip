// Offline derivation of the non-uniform datatype (paper Sec. 3.3, Eq. (1), with the s_i^2 weighting of
// the appendix on per-channel scaling): the 2^b signposts that minimise
//     sum_i w_i (x_i - Q(x_i))^2,   w_i = F_ii s_i^2,   x = normalised calibration activations,
// found with Lloyd's k-means iteration in one dimension.
//
// Design (gfx950).  An iteration streams the n values and weights once (8 bytes per element: the pass
// is HBM-bound for large n) and needs, per signpost, the sums of w and of w*x over the elements nearest
// to it.  The index of the nearest signpost is data dependent, so the running sums cannot live in
// registers; every lane owns a private column of fp64 accumulators in LDS ([signpost][lane]: no
// atomics, no bank conflicts beyond what 64-bit accesses cost anyway).  Workgroups write their sums to
// a workspace, and a one-workgroup kernel adds them in a fixed order and moves the signposts, which
// stay on the device between iterations.  fp32 distances with ties to the smaller index decide the
// assignment; sums are fp64 (w*x of two fp32 numbers is exact in fp64).
#include <algorithm>
#include "kvq_common.hpp"

namespace {

constexpr int CAL_NT = 256;
constexpr int CAL_MAX_WGS = 2048;
constexpr int CAL_PARTS = 16;            // partial sums per signpost in the update kernel

template <int K>
__device__ __forceinline__ int cal_nearest(const float (&c)[K], float x)
{
    int best = 0;
    float bestd = __builtin_fabsf(x - c[0]);
#pragma unroll
    for (int j = 1; j < K; ++j) {
        const float d = __builtin_fabsf(x - c[j]);
        if (d < bestd) { bestd = d; best = j; }
    }
    return best;
}

// partial[workgroup][K][2] = (sum of w, sum of w*x) over the workgroup's elements nearest to signpost j
template <int K>
__global__ __launch_bounds__(CAL_NT) void kvq_calib_assign(const float *__restrict__ x, const float *__restrict__ w,
                                                           int64_t n, const float *__restrict__ cent,
                                                           double *__restrict__ partial)
{
    __shared__ double acc_w[K][CAL_NT], acc_wx[K][CAL_NT];
    const int tid = threadIdx.x;
    float c[K];
#pragma unroll
    for (int j = 0; j < K; ++j) {
        c[j] = cent[j];
        acc_w[j][tid] = 0.0;
        acc_wx[j][tid] = 0.0;
    }
    // groups of four consecutive elements per lane (16-byte loads), grid-stride over the groups
    const int64_t n4 = n >> 2;
    const float4 *x4 = (const float4 *)x, *w4 = (const float4 *)w;
    for (int64_t g = (int64_t)blockIdx.x * CAL_NT + tid; g < n4; g += (int64_t)gridDim.x * CAL_NT) {
        const float4 xv = x4[g], wv = w4[g];
        const float xs[4] = {xv.x, xv.y, xv.z, xv.w}, ws[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = cal_nearest<K>(c, xs[e]);
            const double wd = (double)ws[e];
            acc_w[j][tid] += wd;
            acc_wx[j][tid] += wd * (double)xs[e];
        }
    }
    // the last n % 4 elements
    if (blockIdx.x == 0 && tid < (int)(n & 3)) {
        const int64_t i = (n4 << 2) + tid;
        const int j = cal_nearest<K>(c, x[i]);
        const double wd = (double)w[i];
        acc_w[j][tid] += wd;
        acc_wx[j][tid] += wd * (double)x[i];
    }
    __syncthreads();
    // columns are added up in lane order: thread t < 2K takes one (signpost, sum) row
    if (tid < 2 * K) {
        const int j = tid >> 1;
        const double *row = (tid & 1) ? acc_wx[j] : acc_w[j];
        double s = 0.0;
        for (int l = 0; l < CAL_NT; ++l) s += row[l];
        partial[((int64_t)blockIdx.x * K + j) * 2 + (tid & 1)] = s;
    }
}

// cent[j] = fp32(sum w x / sum w) over all workgroups' partial sums, in a fixed order; a signpost
// whose elements weigh nothing stays where it is
template <int K>
__global__ __launch_bounds__(CAL_PARTS * 16) void kvq_calib_update(const double *__restrict__ partial, int n_wgs,
                                                                   float *__restrict__ cent)
{
    __shared__ double sw[CAL_PARTS][16], swx[CAL_PARTS][16];
    const int j = threadIdx.x & 15, part = threadIdx.x >> 4;
    double a = 0.0, b = 0.0;
    if (j < K) {
        for (int g = part; g < n_wgs; g += CAL_PARTS) {
            a += partial[((int64_t)g * K + j) * 2];
            b += partial[((int64_t)g * K + j) * 2 + 1];
        }
    }
    sw[part][j] = a;
    swx[part][j] = b;
    __syncthreads();
    if (part == 0 && j < K) {
        double ta = 0.0, tb = 0.0;
        for (int p = 0; p < CAL_PARTS; ++p) { ta += sw[p][j]; tb += swx[p][j]; }
        if (ta > 0.0) cent[j] = (float)(tb / ta);
    }
}

template <int K>
kvq_status run_calibration(const float *x, const float *w, int64_t n, int iters, float *cent, double *partial,
                           hipStream_t s)
{
    // enough workgroups to fill the chip (LDS allows 10 / 5 / 2 per compute unit for 4 / 8 / 16
    // signposts), no more than there are groups of 1024 elements, within the workspace's slots
    int64_t wgs = (n / 4 + CAL_NT - 1) / CAL_NT;
    const int64_t fill = 256 * (K == 16 ? 2 : K == 8 ? 5 : 8);
    if (wgs > fill) wgs = fill;
    if (wgs > CAL_MAX_WGS) wgs = CAL_MAX_WGS;
    if (wgs < 1) wgs = 1;
    for (int it = 0; it < iters; ++it) {
        kvq_calib_assign<K><<<(unsigned)wgs, CAL_NT, 0, s>>>(x, w, n, cent, partial);
        kvq_calib_update<K><<<1, CAL_PARTS * 16, 0, s>>>(partial, (int)wgs, cent);
    }
    KVQ_HIP_CHECK(hipGetLastError());
    return KVQ_OK;
}

}  // namespace

extern "C" int64_t kvq_calibrate_workspace_bytes(void)
{
    return (int64_t)CAL_MAX_WGS * 16 * 2 * (int64_t)sizeof(double) + 256;
}

extern "C" kvq_status kvq_calibrate_nuq(const float *d_x_norm, const float *d_w, int64_t n, int32_t bits,
                                        int32_t iters, float *h_signposts, void *d_workspace,
                                        int64_t workspace_bytes, void *stream)
{
    if (!d_x_norm || !d_w || !h_signposts || !d_workspace) return KVQ_ERR_INVALID_ARG;
    if (((uintptr_t)d_x_norm & 15) || ((uintptr_t)d_w & 15) || ((uintptr_t)d_workspace & 255)) return KVQ_ERR_INVALID_ARG;
    if (n < 1 || iters < 0) return KVQ_ERR_INVALID_ARG;
    if (bits < 2 || bits > 4) return KVQ_ERR_UNSUPPORTED;
    if (workspace_bytes < kvq_calibrate_workspace_bytes()) return KVQ_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    const int K = 1 << bits;
    float *cent = (float *)d_workspace;                       // 16 floats, then the partial sums
    double *partial = (double *)((char *)d_workspace + 256);
    KVQ_HIP_CHECK(hipMemcpyAsync(cent, h_signposts, (size_t)K * sizeof(float), hipMemcpyHostToDevice, s));
    kvq_status st = (bits == 2)   ? run_calibration<4>(d_x_norm, d_w, n, iters, cent, partial, s)
                    : (bits == 3) ? run_calibration<8>(d_x_norm, d_w, n, iters, cent, partial, s)
                                  : run_calibration<16>(d_x_norm, d_w, n, iters, cent, partial, s);
    if (st != KVQ_OK) return st;
    KVQ_HIP_CHECK(hipMemcpyAsync(h_signposts, cent, (size_t)K * sizeof(float), hipMemcpyDeviceToHost, s));
    KVQ_HIP_CHECK(hipStreamSynchronize(s));
    std::sort(h_signposts, h_signposts + K);
    return KVQ_OK;
}
