// Online quantize-and-append of new Key / Value vectors (paper Sec. 3.1, 3.4, 3.6, 3.7).
//
// One workgroup per new token.  Every fp32 step is a single explicitly rounded operation
// (this file is compiled with floating-point contraction off) so that codes, outlier indices
// and fp16 residuals are reproducible bit for bit.
#include "kvq_common.hpp"
#include "kvq_qk_sparse.hpp"
#include <type_traits>

namespace {

// Measured on 4096-channel tokens with the workgroup-per-token bodies: 1024-thread workgroups finish
// a call of up to 256 tokens in one round (Values: 25 us against 37 us with 256 threads), break even
// at 512 tokens and lose beyond (4096 tokens: 216 us against 105 us), where eight small workgroups
// per compute unit hide each other's barriers.  Values of 1024, 2048 or 4096 channels take the
// four-wavefront body (v_quant_token4) at every call size instead, those of 5120, 6656 or 8192
// channels (40, 52, 64 heads) in bulk appends.
constexpr int KVQ_BULK_TOKENS = 512;      // calls with at least this many tokens count as bulk appends
constexpr int KVQ_KV_SPLIT_TOKENS = 256;  // from here on the combined call runs the Key and Value kernels in turn
constexpr int KVQ_WAVE_TOKENS = 1024;     // Key appends of at least this many tokens: one wavefront per token

// Workgroups have NT threads: 256 for narrow models, 1024 once a token vector has >= 2048 channels
// (fewer passes over the vector, hence fewer barriers, for the single-token decode append).

// Exclusive rank of this thread's flag among all flags of the workgroup, in thread order, plus
// the workgroup total.  `wave_tot` is a shared array of NT/64 words.  Contains two barriers.
template <int NT>
__device__ inline uint32_t block_rank(bool flag, uint32_t *wave_tot, uint32_t &total)
{
    constexpr int NW = NT / 64;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    unsigned long long b = __ballot(flag);
    uint32_t prefix = __popcll(b & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[w] = __popcll(b);
    __syncthreads();
    uint32_t before = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        uint32_t t = wave_tot[i];
        if (i < w) before += t;
        tot += t;
    }
    __syncthreads();
    total = tot;
    return before + prefix;
}

// Number of Key outliers of each new token (threshold test only).  One wavefront per token, eight
// channels per lane and pass (16-byte loads of the fp16 vector, D is a multiple of 128): no barriers.
constexpr int KVQ_COUNT_NT = 256;
__global__ __launch_bounds__(KVQ_COUNT_NT) void kvq_k_count(const void *params, int D, int T, const uint16_t *k_new,
                                                            uint32_t *cnt)
{
    KvqParamsView pv = kvq_params_view(params, D);
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * (KVQ_COUNT_NT / 64) + (threadIdx.x >> 6);
    if (t >= T) return;
    const uint4 *row = (const uint4 *)(k_new + (int64_t)t * D);
    const float4 *lo4 = (const float4 *)pv.lo, *hi4 = (const float4 *)pv.hi;
    uint32_t mine = 0;
    if ((uintptr_t)k_new & 15) {          // input not 16-byte aligned: one channel per lane and pass
        for (int c = lane; c < D; c += 64) {
            const float x = kvq_h2f(k_new[(int64_t)t * D + c]);
            mine += ((x < pv.lo[c]) | (x > pv.hi[c])) ? 1u : 0u;
        }
    } else for (int v = lane; v < D / 8; v += 64) {
        const uint4 h = row[v];
        const float4 la = lo4[2 * v], lb = lo4[2 * v + 1], ha = hi4[2 * v], hb = hi4[2 * v + 1];
        const uint32_t w[4] = {h.x, h.y, h.z, h.w};
        const float lo[8] = {la.x, la.y, la.z, la.w, lb.x, lb.y, lb.z, lb.w};
        const float hi[8] = {ha.x, ha.y, ha.z, ha.w, hb.x, hb.y, hb.z, hb.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float x = kvq_h2f((uint16_t)(w[e >> 1] >> (16 * (e & 1))));
            mine += ((x < lo[e]) | (x > hi[e])) ? 1u : 0u;
        }
    }
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
    if (lane == 0) cnt[t] = mine;
}

// ptr[n0+1+t] = min(ptr[n0] + cnt[0] + ... + cnt[t], cap_nnz); one workgroup, T <= 4096.
__global__ __launch_bounds__(1024) void kvq_ptr_scan(uint32_t *ptr, int64_t n0, int T, const uint32_t *cnt,
                                                     int64_t cap_nnz, int32_t *d_status)
{
    __shared__ uint32_t part[1024];
    const int tid = threadIdx.x;
    uint32_t v[4], s = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int t = tid * 4 + j;
        v[j] = (t < T) ? cnt[t] : 0u;
        s += v[j];
    }
    part[tid] = s;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        uint32_t add = (tid >= o) ? part[tid - o] : 0u;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    uint64_t run = (uint64_t)ptr[n0] + (part[tid] - s);
    bool over = false;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int t = tid * 4 + j;
        run += v[j];
        if (t < T) {
            uint64_t p = run;
            if (p > (uint64_t)cap_nnz) { p = (uint64_t)cap_nnz; over = true; }
            ptr[n0 + 1 + t] = (uint32_t)p;
        }
    }
    if (over) atomicExch(d_status, (int32_t)KVQ_ERR_NNZ_OVERFLOW);
}

// OR one field of `width` bits into a little-endian bit stream held as dwords in shared memory.
__device__ inline void stream_or(uint32_t *words, int bit, uint32_t value, int width)
{
    int w = bit >> 5, sh = bit & 31;
    atomicOr(&words[w], value << sh);
    if (sh + width > 32) atomicOr(&words[w + 1], value >> (32 - sh));
}

// Exclusive ranks, in channel order, of IT flags per thread (flag j belongs to channel block j, a
// block being NT consecutive channels, one per thread): rank[j] counts the set flags of all earlier
// blocks plus those of lower threads in block j.  `wave_tot` is a shared array of IT*NT/64 words.
// Returns the total.  Contains two barriers, whatever IT.
template <int NT, int IT>
__device__ inline uint32_t block_rank_multi(const bool (&flag)[IT], uint32_t (&rank)[IT], uint32_t *wave_tot)
{
    constexpr int NW = NT / 64;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t prefix[IT];
#pragma unroll
    for (int j = 0; j < IT; ++j) {
        const unsigned long long b = __ballot(flag[j]);
        prefix[j] = __popcll(b & ((1ull << lane) - 1ull));
        if (lane == 0) wave_tot[j * NW + w] = __popcll(b);
    }
    __syncthreads();
    uint32_t run = 0;
#pragma unroll
    for (int j = 0; j < IT; ++j) {
        uint32_t before = 0, tot = 0;
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const uint32_t t = wave_tot[j * NW + i];
            if (i < w) before += t;
            tot += t;
        }
        rank[j] = run + before + prefix[j];
        run += tot;
    }
    __syncthreads();
    return run;
}

// Quantize, pack and append the Keys of one new token per workgroup.
// If `single` the token's outlier count is written to ptr[n+1] here; otherwise ptr[] was already
// filled by kvq_ptr_scan and is only read.
// A pass handles IT blocks of NT channels: all its loads are issued up front, and ranks, packing and
// stores of the IT blocks share one set of barriers (a single-token decode append is pure latency).
// (The body of the kernels below: `t` is the token's index within the call.)
template <int BITS, int NT, class SP>
__device__ __forceinline__ void k_quant_token(const void *__restrict__ params, int D, int64_t cap, int64_t n0,
                                              const uint16_t *__restrict__ k_new, uint8_t *__restrict__ k_codes,
                                              uint32_t *__restrict__ k_ptr, const SP ksp, int64_t cap_nnz, int single,
                                              int32_t *d_status, const int t)
{
    constexpr int NE = 1 << BITS;
    constexpr int CW = 4 * BITS;                 // dwords per chunk
    constexpr int NW = NT / 64;
    constexpr int HB = NT / KVQ_HEAD_DIM;        // heads covered by one block of NT channels
    constexpr int IT = 4;                        // blocks per pass
    __shared__ uint8_t codes_s[IT][NT];
    __shared__ uint32_t chunk_s[IT][HB][CW + 1];
    __shared__ uint32_t wave_tot[IT * NW];
    KvqParamsView pv = kvq_params_view(params, D);
    float lut[NE];
#pragma unroll
    for (int j = 0; j < NE; ++j) lut[j] = pv.hdr->lut_k[j];

    const int tid = threadIdx.x;
    const int64_t n = n0 + t;
    const uint32_t base = k_ptr[n];
    uint32_t running = 0;
    bool overflow = false;
    for (int cb = 0; cb < D; cb += NT * IT) {
        bool is_out[IT];
        uint16_t resid[IT];
        // every load of the pass first (no short-circuit evaluation below: a conditional load would
        // wait for the ones before it), then the arithmetic
        uint16_t xb[IT];
        float zc[IT], sc[IT], ri[IT], lo[IT], hi[IT];
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int c = cb + j * NT + tid;
            const int cc = (c < D) ? c : D - 1;                      // clamped: straight-line loads
            xb[j] = k_new[(int64_t)t * D + cc];
            zc[j] = pv.z[cc]; sc[j] = pv.s[cc]; ri[j] = pv.rinv[cc]; lo[j] = pv.lo[cc]; hi[j] = pv.hi[cc];
        }
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int c = cb + j * NT + tid;
            const float x = kvq_h2f(xb[j]);
            const float diff = x - zc[j];
            const float xn = diff * ri[j];
            float sp;
            const int code = kvq_nearest<NE>(lut, xn, sp);
            const float deq = __builtin_fmaf(sc[j], sp, zc[j]);
            is_out[j] = (c < D) & ((x < lo[j]) | (x > hi[j]));
            resid[j] = kvq_f2h_rn(x - deq);
            codes_s[j][tid] = (uint8_t)code;
        }
        for (int i = tid; i < IT * HB * (CW + 1); i += NT) (&chunk_s[0][0][0])[i] = 0;
        uint32_t rank[IT];
        const uint32_t tot = block_rank_multi<NT, IT>(is_out, rank, wave_tot);   // barriers inside
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            if (is_out[j]) {
                const uint64_t pos = (uint64_t)base + running + rank[j];
                if (pos < (uint64_t)cap_nnz) ksp.put(pos, (uint16_t)(cb + j * NT + tid), resid[j]);
                else overflow = true;
            }
        }
        running += tot;
        // pack the heads covered by each block of NT channels
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int c0 = cb + j * NT;
            const int heads_here = (c0 >= D) ? 0 : ((D - c0 >= NT) ? HB : (D - c0) / KVQ_HEAD_DIM);
            if (tid < 64 * heads_here) {
                const int hh = tid >> 6, i = tid & 63;
                const uint32_t field = (uint32_t)codes_s[j][hh * 128 + i] | ((uint32_t)codes_s[j][hh * 128 + i + 64] << BITS);
                stream_or(chunk_s[j][hh], i * 2 * BITS, field, 2 * BITS);
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int c0 = cb + j * NT;
            const int heads_here = (c0 >= D) ? 0 : ((D - c0 >= NT) ? HB : (D - c0) / KVQ_HEAD_DIM);
            if (tid < CW * heads_here) {
                const int hh = tid / CW, wd = tid % CW;
                const int64_t off = kvq_k_piece0(BITS, cap, n, c0 / KVQ_HEAD_DIM + hh) + (wd >> 2) * 1024 + (wd & 3) * 4;
                *(uint32_t *)(k_codes + off) = chunk_s[j][hh][wd];
            }
        }
        if (cb + NT * IT < D) __syncthreads();       // the next pass reuses the shared arrays
    }
    if (single && tid == 0) {
        uint64_t p = (uint64_t)base + running;
        k_ptr[n + 1] = (uint32_t)(p > (uint64_t)cap_nnz ? (uint64_t)cap_nnz : p);
    }
    if (overflow || (single && tid == 0 && (uint64_t)base + running > (uint64_t)cap_nnz))
        atomicExch(d_status, (int32_t)KVQ_ERR_NNZ_OVERFLOW);
}

// ---- Values -------------------------------------------------------------------------------

// Order-preserving 16-bit key of an fp16 bit pattern (-0 is treated as +0).
__device__ inline uint32_t order_key(uint16_t h)
{
    if (h == 0x8000u) h = 0;
    return (h & 0x8000u) ? (uint32_t)(uint16_t)~h : (uint32_t)(h | 0x8000u);
}

// For the 256 histogram bins held one per thread (threads >= 256 pass 0): the number of elements in
// bins strictly above this thread's bin.  Suffix scan inside each wavefront plus the totals of the
// (up to four) wavefronts that hold bins.  `wsum` is a shared array of 4 words.  One barrier.
__device__ inline uint32_t bins_above(uint32_t mine, uint32_t *wsum)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t s = mine;                            // becomes the sum over lanes lane..63
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_down(s, o);
        if (lane + o < 64) s += t;
    }
    if (lane == 0 && w < 4) wsum[w] = s;
    __syncthreads();
    uint32_t above = s - mine;
    for (int i = w + 1; i < 4; ++i) above += wsum[i];
    return above;
}

// Workgroup-wide selection of the `k` largest keys among elements with state[c]==0, where the key
// of element c is keys[c] ^ flip (flip = 0xFFFF turns it into a selection of the k smallest).
// Marks the selected elements with `mark`; equal keys are taken in ascending index order.
// Two-level radix select on the 16-bit keys; the index-ordered pass over the elements equal to the
// threshold is only needed when some but not all of them are taken.
template <int NT>
__device__ void select_top(const uint16_t *keys, uint8_t *state, int D, int k, uint32_t flip, uint8_t mark,
                           uint32_t *hist, uint32_t *sh, uint32_t *wave_tot)
{
    const int tid = threadIdx.x;
    // level 1: high byte
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int c = tid; c < D; c += NT)
        if (state[c] == 0) atomicAdd(&hist[((keys[c] ^ flip) & 0xFFFFu) >> 8], 1u);
    __syncthreads();
    {
        const uint32_t mine = (tid < 256) ? hist[tid] : 0u;
        const uint32_t above = bins_above(mine, sh + 4);      // elements in bins strictly above bin `tid`
        if (tid < 256 && above < (uint32_t)k && above + mine >= (uint32_t)k) { sh[0] = tid; sh[1] = above; }
    }
    __syncthreads();
    const uint32_t bin_hi = sh[0], above_hi = sh[1];
    __syncthreads();
    // level 2: low byte inside the selected high bin
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int c = tid; c < D; c += NT) {
        uint32_t key = (keys[c] ^ flip) & 0xFFFFu;
        if (state[c] == 0 && (key >> 8) == bin_hi) atomicAdd(&hist[key & 255u], 1u);
    }
    __syncthreads();
    {
        const uint32_t mine = (tid < 256) ? hist[tid] : 0u;
        const uint32_t above = above_hi + bins_above(mine, sh + 4);
        if (tid < 256 && above < (uint32_t)k && above + mine >= (uint32_t)k) {
            sh[0] = (bin_hi << 8) | tid; sh[1] = above; sh[2] = mine;
        }
    }
    __syncthreads();
    const uint32_t tau = sh[0];
    const uint32_t need_eq = (uint32_t)k - sh[1];  // how many elements equal to tau are taken
    const bool all_eq = need_eq == sh[2];          // ... all of them: no index order needed
    __syncthreads();
    if (all_eq) {
        for (int c = tid; c < D; c += NT)
            if (state[c] == 0 && ((keys[c] ^ flip) & 0xFFFFu) >= tau) state[c] = mark;
    } else {
        uint32_t running = 0;
        for (int c0 = 0; c0 < D; c0 += NT) {
            const int c = c0 + tid;
            bool cand = false, eq = false, gt = false;
            if (c < D && state[c] == 0) {
                uint32_t key = (keys[c] ^ flip) & 0xFFFFu;
                gt = key > tau;
                eq = key == tau;
                cand = true;
            }
            uint32_t tot;
            uint32_t rank = running + block_rank<NT>(eq, wave_tot, tot);
            running += tot;
            if (cand && (gt || (eq && rank < need_eq))) state[c] = mark;
        }
    }
    __syncthreads();
}

// Two bin sets at once (same scan as bins_above, one barrier for both).  `wsum` holds 8 words.
__device__ inline void bins_above2(uint32_t mine_a, uint32_t mine_b, uint32_t *wsum, uint32_t &above_a,
                                   uint32_t &above_b)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t sa = mine_a, sb = mine_b;
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t ta = __shfl_down(sa, o), tb = __shfl_down(sb, o);
        if (lane + o < 64) { sa += ta; sb += tb; }
    }
    if (lane == 0 && w < 4) { wsum[w] = sa; wsum[4 + w] = sb; }
    __syncthreads();
    above_a = sa - mine_a;
    above_b = sb - mine_b;
    for (int i = w + 1; i < 4; ++i) { above_a += wsum[i]; above_b += wsum[4 + i]; }
}

// The k largest keys (marked 1) and, among the rest, the k smallest (marked 2) in one go; state[] is
// all zero on entry and 2k < D.  Equal keys are taken in ascending index order on both sides.  Both
// thresholds come out of the same two histogram passes (high byte, then low byte inside the two
// selected bins).  Because 2k < D the k-th largest key is >= the k-th smallest; when they differ the
// two selections cannot interact and this routine is exact; when they coincide (heavy ties) it
// leaves state[] untouched and returns false, and the caller runs the two selections one after the
// other.  hist: 768 words that the caller has cleared (and made visible with a barrier), sh: 24
// words, wave_tot: 2*NT/64 words.
template <int NT>
__device__ bool select_both(const uint16_t *keys, uint8_t *state, int D, int k, uint32_t *hist, uint32_t *sh,
                            uint32_t *wave_tot)
{
    const int tid = threadIdx.x;
    const uint32_t K = (uint32_t)k;
    for (int c = tid; c < D; c += NT) atomicAdd(&hist[keys[c] >> 8], 1u);
    __syncthreads();
    {
        const uint32_t mine = (tid < 256) ? hist[tid] : 0u;
        const uint32_t above = bins_above(mine, sh + 16);
        const uint32_t below = (uint32_t)D - above - mine;
        if (tid < 256 && above < K && above + mine >= K) { sh[0] = tid; sh[1] = above; }
        if (tid < 256 && below < K && below + mine >= K) { sh[2] = tid; sh[3] = below; sh[4] = mine; }
    }
    __syncthreads();
    const uint32_t bin_top = sh[0], above_top = sh[1], bin_bot = sh[2], below_bot = sh[3], in_bot = sh[4];
    for (int c = tid; c < D; c += NT) {
        const uint32_t key = keys[c];
        if ((key >> 8) == bin_top) atomicAdd(&hist[256 + (key & 255u)], 1u);
        if ((key >> 8) == bin_bot) atomicAdd(&hist[512 + (key & 255u)], 1u);
    }
    __syncthreads();
    {
        const uint32_t mt = (tid < 256) ? hist[256 + tid] : 0u, mb = (tid < 256) ? hist[512 + tid] : 0u;
        uint32_t at, ab;
        bins_above2(mt, mb, sh + 16, at, ab);
        const uint32_t above = above_top + at;                   // keys strictly greater than this one
        const uint32_t below = below_bot + (in_bot - ab - mb);   // keys strictly smaller than this one
        if (tid < 256 && above < K && above + mt >= K) { sh[5] = (bin_top << 8) | tid; sh[6] = above; sh[7] = mt; }
        if (tid < 256 && below < K && below + mb >= K) { sh[8] = (bin_bot << 8) | tid; sh[9] = below; sh[10] = mb; }
    }
    __syncthreads();
    const uint32_t tau_top = sh[5], tau_bot = sh[8];
    const uint32_t need_top = K - sh[6], need_bot = K - sh[9];
    const bool all_top = need_top == sh[7], all_bot = need_bot == sh[10];
    if (tau_top == tau_bot) return false;
    if (all_top && all_bot) {
        for (int c = tid; c < D; c += NT) {
            const uint32_t key = keys[c];
            if (key >= tau_top) state[c] = 1;
            else if (key <= tau_bot) state[c] = 2;
        }
    } else {
        // ties straddle a threshold: equal keys are taken in index order
        uint32_t run_top = 0, run_bot = 0;
        for (int c0 = 0; c0 < D; c0 += NT) {
            const int c = c0 + tid;
            const uint32_t key = (c < D) ? keys[c] : 0u;
            const bool flag[2] = {c < D && key == tau_top, c < D && key == tau_bot};
            uint32_t rank[2];
            // ranks of flag[1] continue after all of flag[0]: take the per-flag counts apart again
            const uint32_t both = block_rank_multi<NT, 2>(flag, rank, wave_tot);
            const uint32_t n_top = __syncthreads_count(flag[0]);
            const uint32_t rt = run_top + rank[0], rb = run_bot + (rank[1] - n_top);
            if (c < D) {
                if (key > tau_top || (flag[0] && rt < need_top)) state[c] = 1;
                else if (key < tau_bot || (flag[1] && rb < need_bot)) state[c] = 2;
            }
            run_top += n_top;
            run_bot += both - n_top;
        }
    }
    __syncthreads();
    return true;
}

// Quantize, pack and append the Values of one new token per workgroup (`t`: the token's index within
// the call).  A pass of the main loop handles IT blocks of NT channels (see k_quant_token).
template <int BITS, int NT, class SP>
__device__ __forceinline__ void v_quant_token(const void *__restrict__ params, int D, int64_t cap, int64_t n0,
                                              int k_side, const uint16_t *__restrict__ v_new,
                                              uint8_t *__restrict__ v_codes, uint16_t *__restrict__ v_sz,
                                              uint32_t *__restrict__ v_ptr, const SP vsp, int64_t cap_nnz, int32_t *d_status,
                                              const int t)
{
    constexpr int NE = 1 << BITS;
    constexpr int CW = 4 * BITS;
    constexpr int IT = 4;                         // blocks per pass
    extern __shared__ uint8_t dyn[];              // keys: 2*D bytes, state: D bytes
    uint16_t *keys = (uint16_t *)dyn;
    uint8_t *state = dyn + 2 * (size_t)D;
    constexpr int NW = NT / 64;
    constexpr int CB = NT / 64;                   // (head, half) chunks covered by one block of NT channels
    __shared__ uint32_t hist[768];
    __shared__ uint32_t sh[24];
    __shared__ uint32_t wave_tot[IT * NW];
    __shared__ float redmx[NW], redmn[NW];
    __shared__ uint8_t codes_s[IT][NT];
    __shared__ uint32_t bits_s[IT][CB][CW + 1], mask_s[IT][CB][CW + 1];

    KvqParamsView pv = kvq_params_view(params, D);
    float lut[NE];
#pragma unroll
    for (int j = 0; j < NE; ++j) lut[j] = pv.hdr->lut_v[j];
    const int tid = threadIdx.x;
    const int64_t n = n0 + t;
    const uint16_t *x16 = v_new + (int64_t)t * D;
    const uint32_t base = v_ptr[n0] + (uint32_t)t * 2u * (uint32_t)k_side;

    // The thread's first IT elements (channels tid, tid + NT, ...) stay in registers for the later
    // passes; wider vectors re-read the rest from memory.
    uint16_t xc[IT];
#pragma unroll
    for (int j = 0; j < IT; ++j) {
        const int c = tid + j * NT;
        xc[j] = x16[c < D ? c : D - 1];
    }
#pragma unroll
    for (int j = 0; j < IT; ++j) {
        const int c = tid + j * NT;
        if (c < D) { keys[c] = (uint16_t)order_key(xc[j]); state[c] = 0; }
    }
    for (int c = tid + IT * NT; c < D; c += NT) { keys[c] = (uint16_t)order_key(x16[c]); state[c] = 0; }
    for (int i = tid; i < 768; i += NT) hist[i] = 0;   // the three histograms of select_both
    __syncthreads();
    if (k_side > 0) {
        if (!select_both<NT>(keys, state, D, k_side, hist, sh, wave_tot)) {
            select_top<NT>(keys, state, D, k_side, 0u, 1, hist, sh, wave_tot);        // k largest
            select_top<NT>(keys, state, D, k_side, 0xFFFFu, 2, hist, sh, wave_tot);   // k smallest of the rest
        }
    }
    // range of the remaining elements
    float mx = -INFINITY, mn = INFINITY;
#pragma unroll
    for (int j = 0; j < IT; ++j) {
        const int c = tid + j * NT;
        if (c < D && state[c] == 0) { float x = kvq_h2f(xc[j]); mx = fmaxf(mx, x); mn = fminf(mn, x); }
    }
    for (int c = tid + IT * NT; c < D; c += NT)
        if (state[c] == 0) { float x = kvq_h2f(x16[c]); mx = fmaxf(mx, x); mn = fminf(mn, x); }
    for (int o = 32; o > 0; o >>= 1) { mx = fmaxf(mx, __shfl_xor(mx, o)); mn = fminf(mn, __shfl_xor(mn, o)); }
    if ((tid & 63) == 0) { redmx[tid >> 6] = mx; redmn[tid >> 6] = mn; }
    __syncthreads();
    mx = redmx[0]; mn = redmn[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) { mx = fmaxf(mx, redmx[i]); mn = fminf(mn, redmn[i]); }
    const float sum = mx + mn, dif = mx - mn;
    uint16_t zb = kvq_f2h_rn(sum * 0.5f), sb = kvq_f2h_rn(dif * 0.5f);
    float zf = kvq_h2f(zb), sf = kvq_h2f(sb);
    if (sf == 0.0f) { sf = 1.0f; sb = 0x3c00u; }
    const float rinv = __fdiv_rn(1.0f, sf);
    if (tid == 0) { v_sz[n * 2 + 0] = sb; v_sz[n * 2 + 1] = zb; }

    const int parity = (int)(n & 1);
    uint32_t running = 0;
    bool overflow = false;
    for (int cb = 0; cb < D; cb += NT * IT) {
        bool is_out[IT];
        uint16_t resid[IT];
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int c = cb + j * NT + tid;
            const int cc = (c < D) ? c : D - 1;
            const float x = kvq_h2f(cb == 0 ? xc[j] : x16[cc]);      // the first pass has its elements in registers
            const float diff = x - zf;
            const float xn = diff * rinv;
            float sp;
            const int code = kvq_nearest<NE>(lut, xn, sp);
            const float deq = __builtin_fmaf(sf, sp, zf);
            is_out[j] = (c < D) && state[cc] != 0;
            resid[j] = kvq_f2h_rn(x - deq);
            codes_s[j][tid] = (uint8_t)code;
        }
        for (int i = tid; i < IT * CB * (CW + 1); i += NT) { (&bits_s[0][0][0])[i] = 0; (&mask_s[0][0][0])[i] = 0; }
        uint32_t rank[IT];
        const uint32_t tot = block_rank_multi<NT, IT>(is_out, rank, wave_tot);   // barriers inside
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            if (is_out[j]) {
                const uint64_t pos = (uint64_t)base + running + rank[j];
                if (pos < (uint64_t)cap_nnz) vsp.put(pos, (uint16_t)(cb + j * NT + tid), resid[j]);
                else overflow = true;
            }
        }
        running += tot;
        // a block of NT channels covers up to CB (head, half) chunks of 64 fields each
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int c0 = cb + j * NT;
            const int chunks_here = (c0 >= D) ? 0 : ((D - c0 >= NT) ? CB : (D - c0) / 64);
            if (tid < 64 * chunks_here) {
                const int q = tid >> 6, i = tid & 63;
                stream_or(bits_s[j][q], i * 2 * BITS + parity * BITS, (uint32_t)codes_s[j][tid], BITS);
                stream_or(mask_s[j][q], i * 2 * BITS + parity * BITS, (uint32_t)(NE - 1), BITS);
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int c0 = cb + j * NT;
            const int chunks_here = (c0 >= D) ? 0 : ((D - c0 >= NT) ? CB : (D - c0) / 64);
            if (tid < CW * chunks_here) {
                const int q = tid / CW, wd = tid % CW;
                const int ch0 = c0 + q * 64;
                const int64_t off = kvq_v_piece0(BITS, cap, n >> 1, ch0 / KVQ_HEAD_DIM, (ch0 >> 6) & 1) + (wd >> 2) * 1024 + (wd & 3) * 4;
                uint32_t *p = (uint32_t *)(v_codes + off);
                // The partner token of the pair owns the other bits of this dword and may be written
                // concurrently by another workgroup: clear this token's bits, then set them, with two
                // atomics that return nothing (no round trip; the same thread's atomics on one address
                // are applied in order, and the partner's touch disjoint bits).
                __hip_atomic_fetch_and(p, ~mask_s[j][q][wd], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_fetch_or(p, bits_s[j][q][wd], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (cb + NT * IT < D) __syncthreads();     // the next pass reuses the shared arrays
    }
    if (tid == 0) {
        uint64_t p = (uint64_t)base + 2u * (uint32_t)k_side;
        if (p > (uint64_t)cap_nnz) { p = (uint64_t)cap_nnz; overflow = true; }
        v_ptr[n + 1] = (uint32_t)p;
    }
    if (overflow) atomicExch(d_status, (int32_t)KVQ_ERR_NNZ_OVERFLOW);
}

// (256-thread workgroups serve small models and bulk appends: eight wavefronts per SIMD keep more
// tokens in flight; the 1024-thread ones are one workgroup per compute unit anyway)
// Bulk Key append: one wavefront per token, no workgroup barrier.  Lane l takes channels l and l+64
// of every head, the pair that shares a field of the packed chunk, so a head's 64 fields come from the
// 64 lanes; the chunk is assembled in a slice of LDS private to the wavefront.  Outliers keep channel
// order: within a head first the lanes' lower channels, then their upper ones, ranked by ballots.
// Same arithmetic, same results, as k_quant_token; the per-token pointers come from kvq_ptr_scan.
constexpr int KVQ_KW_NT = 256;
template <int BITS, class SP>
__global__ __launch_bounds__(KVQ_KW_NT) void kvq_k_quant_wave(const void *__restrict__ params, int D, int T,
                                                              int64_t cap, int64_t n0,
                                                              const uint16_t *__restrict__ k_new,
                                                              uint8_t *__restrict__ k_codes,
                                                              const uint32_t *__restrict__ k_ptr,
                                                              const SP ksp, int64_t cap_nnz,
                                                              int32_t *d_status)
{
    constexpr int NE = 1 << BITS;
    constexpr int CW = 4 * BITS;                 // dwords per chunk
    __shared__ uint32_t chunk_s[KVQ_KW_NT / 64][CW + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = blockIdx.x * (KVQ_KW_NT / 64) + wave;
    if (t >= T) return;                          // whole wavefronts leave; there is no workgroup barrier below
    KvqParamsView pv = kvq_params_view(params, D);
    float lut[NE];
#pragma unroll
    for (int j = 0; j < NE; ++j) lut[j] = pv.hdr->lut_k[j];
    const int64_t n = n0 + t;
    const uint32_t base = k_ptr[n];
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    uint32_t *chunk = chunk_s[wave];
    uint32_t running = 0;
    bool overflow = false;
    const int H = D / KVQ_HEAD_DIM;
    for (int h = 0; h < H; ++h) {
        const int c0 = h * KVQ_HEAD_DIM + lane, c1 = c0 + 64;
        const uint16_t xb0 = k_new[(int64_t)t * D + c0], xb1 = k_new[(int64_t)t * D + c1];
        const float z0 = pv.z[c0], s0 = pv.s[c0], r0 = pv.rinv[c0], lo0 = pv.lo[c0], hi0 = pv.hi[c0];
        const float z1 = pv.z[c1], s1 = pv.s[c1], r1 = pv.rinv[c1], lo1 = pv.lo[c1], hi1 = pv.hi[c1];
        if (lane <= CW) chunk[lane] = 0;
        const float x0 = kvq_h2f(xb0), x1 = kvq_h2f(xb1);
        float sp0, sp1;
        const float d0 = x0 - z0, d1 = x1 - z1;
        const int code0 = kvq_nearest<NE>(lut, d0 * r0, sp0);
        const int code1 = kvq_nearest<NE>(lut, d1 * r1, sp1);
        const float deq0 = __builtin_fmaf(s0, sp0, z0), deq1 = __builtin_fmaf(s1, sp1, z1);
        const bool o0 = (x0 < lo0) | (x0 > hi0), o1 = (x1 < lo1) | (x1 > hi1);
        // outliers of this head in channel order
        const unsigned long long b0 = __ballot(o0), b1 = __ballot(o1);
        const uint32_t rank0 = running + (uint32_t)__popcll(b0 & lt_mask);
        running += (uint32_t)__popcll(b0);
        const uint32_t rank1 = running + (uint32_t)__popcll(b1 & lt_mask);
        running += (uint32_t)__popcll(b1);
        if (o0) {
            const uint64_t pos = (uint64_t)base + rank0;
            if (pos < (uint64_t)cap_nnz) ksp.put(pos, (uint16_t)c0, kvq_f2h_rn(x0 - deq0));
            else overflow = true;
        }
        if (o1) {
            const uint64_t pos = (uint64_t)base + rank1;
            if (pos < (uint64_t)cap_nnz) ksp.put(pos, (uint16_t)c1, kvq_f2h_rn(x1 - deq1));
            else overflow = true;
        }
        // the head's chunk: 64 fields of 2*BITS bits, assembled in the wavefront's LDS slice (LDS
        // operations of one wavefront execute in order; the fences keep the compiler from reordering them)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        stream_or(chunk, lane * 2 * BITS, (uint32_t)code0 | ((uint32_t)code1 << BITS), 2 * BITS);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (lane < CW) {
            const int64_t off = kvq_k_piece0(BITS, cap, n, h) + (lane >> 2) * 1024 + (lane & 3) * 4;
            *(uint32_t *)(k_codes + off) = chunk[lane];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    if (overflow) atomicExch(d_status, (int32_t)KVQ_ERR_NNZ_OVERFLOW);
}

// ---- bulk Value append -----------------------------------------------------------------------
// In a histogram of 256 bins (lane l reads bins 4l..4l+3), the bin in which the K-th element counted
// from the top (FROM_TOP) or from the bottom lies, the number of elements beyond that bin on that side,
// and the bin's own count.  Wavefront-uniform results.  1 <= K <= number of elements.
template <bool FROM_TOP>
__device__ __forceinline__ void wave_find_bin(const uint32_t *h256, uint32_t K, int lane, uint32_t &bin,
                                              uint32_t &beyond, uint32_t &in_bin)
{
    const uint4 v = *(const uint4 *)(h256 + 4 * lane);
    const uint32_t hh[4] = {v.x, v.y, v.z, v.w};
    const uint32_t s = v.x + v.y + v.z + v.w;
    uint32_t S = s;                                // sum over this lane and the lanes on the side counted from
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = FROM_TOP ? __shfl_down(S, o) : __shfl_up(S, o);
        if (FROM_TOP ? (lane + o < 64) : (lane >= o)) S += t;
    }
    uint32_t a = S - s;                            // elements in the bins of the lanes beyond this one
    int found = -1;
    uint32_t fa = 0, fh = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = FROM_TOP ? 3 - i : i;
        if (found < 0 && a < K && a + hh[q] >= K) { found = q; fa = a; fh = hh[q]; }
        a += hh[q];
    }
    const int src = __ffsll((unsigned long long)__ballot(found >= 0)) - 1;      // exactly one lane finds it
    bin = (uint32_t)__shfl(4 * lane + found, src);
    beyond = __shfl(fa, src);
    in_bin = __shfl(fh, src);
}

// Value append: one workgroup of four wavefronts per token, D = 256 * JW channels (JW = 4, 8, 16,
// 20, 26 or 32).  Wavefront w takes the channel groups j = w JW .. (w + 1) JW - 1, lane l of it the channels
// 64 j + l (half j & 1 of head j >> 1), so a wavefront packs whole chunks on its own, channel order is
// wavefront order, and a lane keeps its JW elements in registers from the one load to the end.  The
// selection is the two-level radix selection of select_both on histograms shared by the four
// wavefronts (each reads the bins it needs itself); equal keys at a threshold are taken in channel
// order, ranked with ballots and the wavefronts' counts, and when the two thresholds coincide the
// upper outliers take the first of the equal keys and the lower ones the next, which is what taking
// the k largest first and then the k smallest of the rest comes to.  The packed codes of all JW chunks
// are gathered in the wavefront's LDS slice and written by all 64 lanes at the end.  Five workgroup
// barriers per token (six when equal keys must be ranked).  Same arithmetic, same results, as
// v_quant_token.
// W wavefronts per token instead of four (D = 64 W JW): the same routine with fewer elements per lane,
// for calls of a few tokens, where the time of a token is the length of a lane's instruction stream
// (a 4096-channel token: 16 elements per lane on four wavefronts, 4 on sixteen).
constexpr int KVQ_VW_WAVES = 4;
constexpr int KVQ_VW_NT = 64 * KVQ_VW_WAVES;
constexpr int KVQ_VW_SMALL_TOKENS = 64;      // calls below this many tokens use one lane per four elements
template <int BITS, int JW, int W, class SP>
__device__ __forceinline__ void v_quant_token4(const void *__restrict__ params, int D, int64_t cap, int64_t n0,
                                               int k_side, const uint16_t *__restrict__ v_new,
                                               uint8_t *__restrict__ v_codes, uint16_t *__restrict__ v_sz,
                                               uint32_t *__restrict__ v_ptr, const SP vsp, int64_t cap_nnz, int32_t *d_status,
                                               const int t)
{
    constexpr int NE = 1 << BITS;
    constexpr int CW = 4 * BITS;
    constexpr int NTW = 64 * W;                  // threads that work on the token
    constexpr int WB = W < 4 ? W : 4;            // wavefronts whose lane extremes bound the thresholds
    __shared__ __attribute__((aligned(16))) uint32_t hist[768];
    __shared__ uint32_t bits_s[W][JW][CW + 1], mask_s[W][CW + 1];
    __shared__ uint32_t eq_cnt[W][2], out_cnt[W];
    __shared__ uint16_t lane_max[NTW], lane_min[NTW];
    __shared__ float red_mx[W], red_mn[W];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t(*bits)[CW + 1] = bits_s[wave];
    uint32_t *mask = mask_s[wave];
    KvqParamsView pv = kvq_params_view(params, D);
    float lut[NE];
#pragma unroll
    for (int j = 0; j < NE; ++j) lut[j] = pv.hdr->lut_v[j];
    const int jb = wave * JW;                    // this wavefront's first channel group (D = 64 W JW)
    const int64_t n = n0 + t;
    const uint16_t *x16 = v_new + (int64_t)t * D + lane;
    const uint32_t base = v_ptr[n0] + (uint32_t)t * 2u * (uint32_t)k_side;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    const uint32_t K = (uint32_t)k_side;

    // the wavefront's packing area, cleared here and filled after the barrier that follows the ranges
    for (int e = lane; e < JW * (CW + 1); e += 64) (&bits[0][0])[e] = 0;
    if (lane <= CW) mask[lane] = 0;
    uint16_t xc[JW];                             // this lane's elements, kept in registers
#pragma unroll
    for (int i = 0; i < JW; ++i) xc[i] = x16[64 * (jb + i)];

    uint32_t top = 0, bot = 0;                   // bit i: channel 64 (jb + i) + lane is an upper / lower outlier
    static_assert(JW <= 32, "one mask bit per element of a lane");
    if (K > 0) {
        for (int i = threadIdx.x; i < 768; i += NTW) hist[i] = 0;
        // Only the tails go into the histograms (shared-memory atomics on the few bins that hold the
        // bulk of a token would serialize).  The K-th largest of the 64 W lanes' largest keys is a lower
        // bound of the K-th largest key of the token, since that many elements are at least as large;
        // likewise for the smallest.  Every wavefront finds both bounds by bisection over the 16 key
        // bits, with ballots.  Histogram counts are then exact from the bounds outwards, which is all
        // the searches below read.  More outliers per side than lanes: no bound, every key counts.
        uint32_t kc[JW];                         // the elements' order-preserving keys
#pragma unroll
        for (int i = 0; i < JW; ++i) kc[i] = order_key(xc[i]);
        uint32_t kmax = 0, kmin = 0xffffu;
#pragma unroll
        for (int i = 0; i < JW; ++i) {
            const uint32_t key = kc[i];
            kmax = key > kmax ? key : kmax;
            kmin = key < kmin ? key : kmin;
        }
        lane_max[threadIdx.x] = (uint16_t)kmax;
        lane_min[threadIdx.x] = (uint16_t)kmin;
        __syncthreads();
        uint32_t m_top = 0, m_bot = 0xffffu;
        if (K <= (uint32_t)(64 * WB)) {
            // (the lanes of the first WB wavefronts are enough: the K-th largest of ANY 64 WB elements
            // of the token is a lower bound of its K-th largest key)
            uint32_t vt[WB], vb[WB];
#pragma unroll
            for (int r = 0; r < WB; ++r) { vt[r] = lane_max[lane + 64 * r]; vb[r] = 0xffffu - lane_min[lane + 64 * r]; }
            uint32_t inv_bot = 0;
            for (int bit = 15; bit >= 0; --bit) {
                const uint32_t ct = m_top | (1u << bit), cb = inv_bot | (1u << bit);
                uint32_t nt = 0, nb = 0;
#pragma unroll
                for (int r = 0; r < WB; ++r) {
                    nt += (uint32_t)__popcll(__ballot(vt[r] >= ct));
                    nb += (uint32_t)__popcll(__ballot(vb[r] >= cb));
                }
                if (nt >= K) m_top = ct;
                if (nb >= K) inv_bot = cb;
            }
            m_bot = 0xffffu - inv_bot;
        }
#pragma unroll
        for (int i = 0; i < JW; ++i) {
            const uint32_t key = kc[i];
            if (key >= m_top || key <= m_bot) atomicAdd(&hist[key >> 8], 1u);
        }
        __syncthreads();
        uint32_t bin_top, above_top, in_top, bin_bot, below_bot, in_bot;
        wave_find_bin<true>(hist, K, lane, bin_top, above_top, in_top);
        wave_find_bin<false>(hist, K, lane, bin_bot, below_bot, in_bot);
#pragma unroll
        for (int i = 0; i < JW; ++i) {
            const uint32_t key = kc[i];
            if ((key >> 8) == bin_top && key >= m_top) atomicAdd(&hist[256 + (key & 255u)], 1u);
            if ((key >> 8) == bin_bot && key <= m_bot) atomicAdd(&hist[512 + (key & 255u)], 1u);
        }
        __syncthreads();
        uint32_t lo_top, above_in, n_eq_top, lo_bot, below_in, n_eq_bot;
        wave_find_bin<true>(hist + 256, K - above_top, lane, lo_top, above_in, n_eq_top);
        wave_find_bin<false>(hist + 512, K - below_bot, lane, lo_bot, below_in, n_eq_bot);
        const uint32_t tau_top = (bin_top << 8) | lo_top, tau_bot = (bin_bot << 8) | lo_bot;
        const uint32_t need_top = K - (above_top + above_in), need_bot = K - (below_bot + below_in);
        const bool same = tau_top == tau_bot;
        // ranks of equal keys are only needed when some but not all of them are taken (wavefront-uniform,
        // and the same in all four wavefronts: the barrier inside is reached by all or none)
        const bool ranked = same || need_top != n_eq_top || need_bot != n_eq_bot;
        uint32_t run_top = 0, run_bot = 0;       // equal keys before this wavefront's channels, then running
        if (ranked) {
            uint32_t ct = 0, cb = 0;
#pragma unroll
            for (int i = 0; i < JW; ++i) {
                const uint32_t key = kc[i];
                ct += (uint32_t)__popcll(__ballot(key == tau_top));
                cb += (uint32_t)__popcll(__ballot(key == tau_bot));
            }
            if (lane == 0) { eq_cnt[wave][0] = ct; eq_cnt[wave][1] = cb; }
            __syncthreads();
            for (int w = 0; w < wave; ++w) { run_top += eq_cnt[w][0]; run_bot += eq_cnt[w][1]; }
        }
#pragma unroll
        for (int i = 0; i < JW; ++i) {
            const uint32_t key = kc[i];
            const bool eq_t = key == tau_top, eq_b = key == tau_bot;
            bool is_top, is_bot;
            if (ranked) {
                const unsigned long long bt = __ballot(eq_t), bb = __ballot(eq_b);
                const uint32_t rt = run_top + (uint32_t)__popcll(bt & lt_mask);
                const uint32_t rb = run_bot + (uint32_t)__popcll(bb & lt_mask);
                run_top += (uint32_t)__popcll(bt);
                run_bot += (uint32_t)__popcll(bb);
                is_top = key > tau_top || (eq_t && rt < need_top);
                // thresholds coincide: the lower outliers take the equal keys that follow the upper ones'
                is_bot = !is_top && (key < tau_bot ||
                                     (eq_b && (same ? (rb >= need_top && rb < need_top + need_bot) : rb < need_bot)));
            } else {
                is_top = key >= tau_top;
                is_bot = key <= tau_bot;
            }
            top |= (uint32_t)is_top << i;
            bot |= (uint32_t)is_bot << i;
        }
    }
    // range of the remaining elements, and this wavefront's number of outliers
    float mx = -INFINITY, mn = INFINITY;
    const uint32_t outl = top | bot;
#pragma unroll
    for (int i = 0; i < JW; ++i)
        if (!((outl >> i) & 1u)) { const float x = kvq_h2f(xc[i]); mx = fmaxf(mx, x); mn = fminf(mn, x); }
    uint32_t n_out = (uint32_t)__popc(outl);
    for (int o = 32; o > 0; o >>= 1) {
        mx = fmaxf(mx, __shfl_xor(mx, o));
        mn = fminf(mn, __shfl_xor(mn, o));
        n_out += __shfl_xor(n_out, o);
    }
    if (lane == 0) { red_mx[wave] = mx; red_mn[wave] = mn; out_cnt[wave] = n_out; }
    __syncthreads();
    mx = red_mx[0]; mn = red_mn[0];
#pragma unroll
    for (int w = 1; w < W; ++w) { mx = fmaxf(mx, red_mx[w]); mn = fminf(mn, red_mn[w]); }
    uint32_t running = 0;                        // outliers before this wavefront's channels, then running
    for (int w = 0; w < wave; ++w) running += out_cnt[w];
    const float sum = mx + mn, dif = mx - mn;
    uint16_t zb = kvq_f2h_rn(sum * 0.5f), sb = kvq_f2h_rn(dif * 0.5f);
    float zf = kvq_h2f(zb), sf = kvq_h2f(sb);
    if (sf == 0.0f) { sf = 1.0f; sb = 0x3c00u; }
    const float rinv = __fdiv_rn(1.0f, sf);
    if (threadIdx.x == 0) { v_sz[n * 2 + 0] = sb; v_sz[n * 2 + 1] = zb; }

    const int parity = (int)(n & 1);
    bool overflow = false;
#pragma unroll
    for (int i = 0; i < JW; ++i) {
        const int j = jb + i;
        const float x = kvq_h2f(xc[i]);
        const float diff = x - zf;
        const float xn = diff * rinv;
        float sp;
        const int code = kvq_nearest<NE>(lut, xn, sp);
        const float deq = __builtin_fmaf(sf, sp, zf);
        const bool is_out = (outl >> i) & 1u;
        const unsigned long long b = __ballot(is_out);
        if (is_out) {
            const uint64_t pos = (uint64_t)base + running + (uint32_t)__popcll(b & lt_mask);
            if (pos < (uint64_t)cap_nnz) vsp.put(pos, (uint16_t)(64 * j + lane), kvq_f2h_rn(x - deq));
            else overflow = true;
        }
        running += (uint32_t)__popcll(b);
        // the chunk of (head j >> 1, half j & 1): this token's bits of 64 fields, gathered in the
        // wavefront's own LDS slice
        stream_or(bits[i], lane * 2 * BITS + parity * BITS, (uint32_t)code, BITS);
    }
    stream_or(mask, lane * 2 * BITS + parity * BITS, (uint32_t)(NE - 1), BITS);
    // LDS operations of one wavefront execute in order; the fence keeps the compiler from moving the
    // reads below above the atomics
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (int e = lane; e < JW * CW; e += 64) {
        const int i = e / CW, d = e - i * CW, j = jb + i;
        const int64_t off = kvq_v_piece0(BITS, cap, n >> 1, j >> 1, j & 1) + (d >> 2) * 1024 + (d & 3) * 4;
        uint32_t *p = (uint32_t *)(v_codes + off);
        // the partner token of the pair owns the other bits of this dword: clear this token's bits, then
        // set them, with two atomics that return nothing (as in v_quant_token)
        __hip_atomic_fetch_and(p, ~mask[d], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_or(p, bits[i][d], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (threadIdx.x == 0) {
        uint64_t p = (uint64_t)base + 2u * (uint32_t)k_side;
        if (p > (uint64_t)cap_nnz) { p = (uint64_t)cap_nnz; overflow = true; }
        v_ptr[n + 1] = (uint32_t)p;
    }
    if (overflow) atomicExch(d_status, (int32_t)KVQ_ERR_NNZ_OVERFLOW);
}

template <int BITS, int JW, int W, class SP>
__global__ __launch_bounds__(64 * W) void kvq_v_quant4(const void *__restrict__ params, int D, int64_t cap,
                                                          int64_t n0, int k_side, const uint16_t *__restrict__ v_new,
                                                          uint8_t *__restrict__ v_codes, uint16_t *__restrict__ v_sz,
                                                          uint32_t *__restrict__ v_ptr, const SP vsp, int64_t cap_nnz,
                                                          int32_t *d_status)
{
    v_quant_token4<BITS, JW, W>(params, D, cap, n0, k_side, v_new, v_codes, v_sz, v_ptr, vsp, cap_nnz, d_status,
                                (int)blockIdx.x);
}

template <int BITS, int NT, class SP>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(NT == 256 ? 8 : 4)))
void kvq_k_quant(const void *__restrict__ params, int D, int64_t cap, int64_t n0,
                                                  const uint16_t *__restrict__ k_new, uint8_t *__restrict__ k_codes,
                                                  uint32_t *__restrict__ k_ptr, const SP ksp, int64_t cap_nnz, int single,
                                                  int32_t *d_status)
{
    k_quant_token<BITS, NT>(params, D, cap, n0, k_new, k_codes, k_ptr, ksp, cap_nnz, single, d_status,
                            (int)blockIdx.x);
}

template <int BITS, int NT, class SP>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(NT == 256 ? 8 : 4)))
void kvq_v_quant(const void *__restrict__ params, int D, int64_t cap, int64_t n0,
                                                  int k_side, const uint16_t *__restrict__ v_new,
                                                  uint8_t *__restrict__ v_codes, uint16_t *__restrict__ v_sz,
                                                  uint32_t *__restrict__ v_ptr, const SP vsp, int64_t cap_nnz, int32_t *d_status)
{
    v_quant_token<BITS, NT>(params, D, cap, n0, k_side, v_new, v_codes, v_sz, v_ptr, vsp, cap_nnz, d_status,
                            (int)blockIdx.x);
}

// Offline calibration of one Key channel per workgroup (paper Sec. 3.6 and the appendix on offline
// calibration): the k smallest and the k largest of the channel's T calibration values are its
// outliers; thresholds are the k-th smallest / largest value, and the values strictly inside give
// the zero-point (mid-range) and scale (half-range).  Same two-level radix selection as for the
// per-token Value outliers, on the channel's column of the [T][D] calibration matrix.
// dyn: keys 2*T bytes, state T bytes.
template <int NT>
__global__ __launch_bounds__(NT) void kvq_calib_channel(const uint16_t *__restrict__ k_cal, int T, int D, int k,
                                                        uint16_t *__restrict__ s_out, uint16_t *__restrict__ z_out,
                                                        uint16_t *__restrict__ lo_out, uint16_t *__restrict__ hi_out)
{
    extern __shared__ uint8_t dyn[];
    uint16_t *keys = (uint16_t *)dyn;
    uint8_t *state = dyn + 2 * (size_t)T;
    __shared__ uint32_t hist[768];
    __shared__ uint32_t sh[24];
    __shared__ uint32_t wave_tot[2 * NT / 64];
    __shared__ uint32_t red[4][NT / 64];
    const int tid = threadIdx.x, c = blockIdx.x;
    for (int t = tid; t < T; t += NT) {
        keys[t] = (uint16_t)order_key(k_cal[(int64_t)t * D + c]);
        state[t] = 0;
    }
    for (int i = tid; i < 768; i += NT) hist[i] = 0;
    __syncthreads();
    if (k > 0) {
        if (!select_both<NT>(keys, state, T, k, hist, sh, wave_tot)) {
            select_top<NT>(keys, state, T, k, 0u, 1, hist, sh, wave_tot);        // k largest
            select_top<NT>(keys, state, T, k, 0xFFFFu, 2, hist, sh, wave_tot);   // k smallest of the rest
        }
    }
    // largest key of the lower outliers, smallest of the upper ones, extremes of the rest
    uint32_t lo_key = 0u, hi_key = 0xFFFFu, in_min = 0xFFFFu, in_max = 0u;
    for (int t = tid; t < T; t += NT) {
        const uint32_t key = keys[t];
        const uint32_t st = state[t];
        if (st == 2) lo_key = key > lo_key ? key : lo_key;
        else if (st == 1) hi_key = key < hi_key ? key : hi_key;
        else { in_min = key < in_min ? key : in_min; in_max = key > in_max ? key : in_max; }
    }
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t a = __shfl_xor(lo_key, o), b = __shfl_xor(hi_key, o), d = __shfl_xor(in_min, o), e = __shfl_xor(in_max, o);
        lo_key = a > lo_key ? a : lo_key;
        hi_key = b < hi_key ? b : hi_key;
        in_min = d < in_min ? d : in_min;
        in_max = e > in_max ? e : in_max;
    }
    if ((tid & 63) == 0) {
        red[0][tid >> 6] = lo_key; red[1][tid >> 6] = hi_key; red[2][tid >> 6] = in_min; red[3][tid >> 6] = in_max;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < NT / 64; ++w) {
            lo_key = red[0][w] > lo_key ? red[0][w] : lo_key;
            hi_key = red[1][w] < hi_key ? red[1][w] : hi_key;
            in_min = red[2][w] < in_min ? red[2][w] : in_min;
            in_max = red[3][w] > in_max ? red[3][w] : in_max;
        }
        // back from the order-preserving key to the fp16 bit pattern
        auto bits_of = [](uint32_t key) { return (uint16_t)((key & 0x8000u) ? (key & 0x7FFFu) : (~key & 0xFFFFu)); };
        const float a = kvq_h2f(bits_of(in_min)), b = kvq_h2f(bits_of(in_max));
        const uint16_t zc = kvq_f2h_rn((b + a) * 0.5f);
        uint16_t sc = kvq_f2h_rn((b - a) * 0.5f);
        if (!(kvq_h2f(sc) > 0.0f)) sc = 0x3C00u;                      // 1.0
        s_out[c] = sc;
        z_out[c] = zc;
        lo_out[c] = (k > 0) ? bits_of(lo_key) : (uint16_t)0xFBFFu;   // -65504
        hi_out[c] = (k > 0) ? bits_of(hi_key) : (uint16_t)0x7BFFu;   // +65504
    }
}

// Keys and Values of the same tokens in one launch: even workgroups take a token's Keys, odd ones its
// Values (a single-token append is pure latency, and the two do not depend on each other).
template <class SP>
struct KvAppendArgs {
    const void *params;
    int D, k_side, single;
    int64_t cap, n0_k, n0_v, cap_nnz_k, cap_nnz_v;
    const uint16_t *k_new, *v_new;
    uint8_t *k_codes, *v_codes;
    uint16_t *v_sz;
    uint32_t *k_ptr, *v_ptr;
    SP ksp, vsp;
    int32_t *d_status;
};
template <int BITS, int NT, class SP>
__global__ __launch_bounds__(NT) void kvq_kv_quant(const KvAppendArgs<SP> a)
{
    const int t = (int)(blockIdx.x >> 1);
    if ((blockIdx.x & 1) == 0)
        k_quant_token<BITS, NT>(a.params, a.D, a.cap, a.n0_k, a.k_new, a.k_codes, a.k_ptr, a.ksp, a.cap_nnz_k,
                                a.single, a.d_status, t);
    else if (a.D == 4096 || a.D == 2048 || a.D == 1024) {
        // the routine with one workgroup per token; wavefronts of the workgroup it does not use end here
        // (a barrier waits only for the wavefronts that have not ended).  A wide workgroup puts sixteen
        // (4096 channels) or eight (2048) wavefronts on the token, a narrow one four.
#define V4(J, WV)                                                                                                \
    do {                                                                                                         \
        if (threadIdx.x >= 64 * (WV)) return;                                                                    \
        v_quant_token4<BITS, J, WV>(a.params, a.D, a.cap, a.n0_v, a.k_side, a.v_new, a.v_codes, a.v_sz, a.v_ptr, \
                                    a.vsp, a.cap_nnz_v, a.d_status, t);                                          \
    } while (0)
        if (NT == 1024) {
            if (a.D == 4096) V4(4, 16);
            else if (a.D == 2048) V4(4, 8);
            else V4(4, 4);
        } else {
            if (a.D == 4096) V4(16, 4);
            else if (a.D == 2048) V4(8, 4);
            else V4(4, 4);
        }
#undef V4
    } else
        v_quant_token<BITS, NT>(a.params, a.D, a.cap, a.n0_v, a.k_side, a.v_new, a.v_codes, a.v_sz, a.v_ptr, a.vsp, a.cap_nnz_v, a.d_status, t);
}

// ---- first launch of a generation step ---------------------------------------------------------
// kvq_decode_step appends one token and then attends over the cache that ends with it.  The append is
// two workgroups of pure latency (12 us), and the attention's first kernel, the sparse Key kernel, needs
// the new token only for the last of its scores: here both run as workgroups of one launch.  Workgroup 0
// quantizes the token's Key (the 256-thread body: 62 registers, so the kernel keeps the sparse
// kernel's eight wavefronts per SIMD) and then adds up the sparse part of the token's own scores from
// the entries it has just stored; workgroup 1 quantizes its Value; the others are the sparse Key
// kernel over the tokens that were there before.
struct StepFrontArgs {
    const void *params;
    int D, n_q_heads, k_side;
    int64_t cap, n;                       // n: tokens in the cache before the step
    int64_t cap_nnz_k, cap_nnz_v;
    const uint16_t *k_new, *v_new;
    uint8_t *k_codes, *v_codes;
    uint16_t *v_sz;
    uint32_t *k_ptr, *v_ptr;
    KvqSparseFlat ksp, vsp;
    int32_t *d_status;
    const float *q_rot;
    float scale;
    float *scores;
    int64_t ld, tokens_per_wave;
};
constexpr int KVQ_STEP_K_NT = 256;        // threads of workgroup 0 that work

// Sparse part of the scores of token a.n, whose entries threads 0 .. KVQ_STEP_K_NT-1 of this workgroup
// have just stored: scale * v * (R_n^T q)_c summed per query head, as the sparse kernel does for the
// other tokens (same arithmetic per entry; 64-bit fixed-point sums in LDS).
template <int R>
__device__ __forceinline__ void qk_sparse_new_token(const StepFrontArgs &a)
{
    extern __shared__ __attribute__((aligned(16))) float sparse_dyn[];
    unsigned long long *S = (unsigned long long *)sparse_dyn;            // [n_q_heads]
    const int tid = threadIdx.x;
    for (int j = tid; j < a.n_q_heads; j += KVQ_STEP_K_NT) S[j] = 0ull;
    // the workgroup's stores of the token's entries and of its end pointer are complete ...
    __threadfence_block();
    __syncthreads();
    // ... and are read back past the vector cache, which may hold the pointer's line from before
    const uint32_t p0 = __hip_atomic_load(a.k_ptr + a.n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t p1 = __hip_atomic_load(a.k_ptr + a.n + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const KvqParamsView pv = kvq_params_view(a.params, a.D);
    for (uint32_t e = p0 + (uint32_t)tid; e < p1; e += KVQ_STEP_K_NT) {
        const uint32_t ch = __hip_atomic_load(a.ksp.idx + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float v = kvq_h2f(__hip_atomic_load(a.ksp.val + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        const uint32_t i = ch & 63u;
        const float rev = rope_rev((float)a.n, pv.hdr->rope_vh[i], pv.hdr->rope_vl[i]);
        const float cs = __builtin_amdgcn_cosf(rev);
        // (R_n^T q)_c = q_c cos + s q_{c^64} sin, s = +1 for the lower channel of the pair, -1 for the upper
        const float sn = __builtin_bit_cast(
            float, __builtin_bit_cast(uint32_t, __builtin_amdgcn_sinf(rev)) ^ ((ch & 64u) << 25));
        const uint32_t cl = ch & 127u, kvh = ch >> 7;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t qh = kvh * R + r, qi = qh * 128u + cl;
            const float qa = a.q_rot[qi] * a.scale, qb = a.q_rot[qi ^ 64u] * a.scale;
            const float qp = qa * cs + qb * sn;
            kvq_lds_add_fixed<0>(&S[qh], v * qp);
        }
    }
    __syncthreads();
    for (int j = tid; j < a.n_q_heads; j += KVQ_STEP_K_NT) a.scores[(int64_t)j * a.ld + a.n] = kvq_from_fixed_fast<0>(S[j]);
}

// W: wavefronts on the Value token (D = 256 W channels: 16 or 4).  One instantiation per width: the
// Value routine's static LDS arrays of several widths would add up and cost the sparse role a workgroup
// per compute unit.
template <int BITS, int R, int W>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8)))
void kvq_step_front(const StepFrontArgs)
{
    // The argument block is read where a role needs it, through a pointer the compiler cannot see
    // through.  Read as a kernel argument it is loaded whole at the kernel's entry, fifty scalar
    // registers that stay alive through all three roles and are spilled into vector-register lanes at
    // once; their reloads (v_readlane) then sit in the sparse role's loops, 25 % more VALU instructions
    // in a role that is bound by them.
#if defined(__HIP_DEVICE_COMPILE__)           // (the host pass only needs the kernel's signature)
    typedef const StepFrontArgs __attribute__((address_space(4))) *ArgsPtr;
    ArgsPtr pa = (ArgsPtr)__builtin_amdgcn_kernarg_segment_ptr();      // the one argument sits at offset 0
    asm volatile("" : "+s"(pa));
    if (blockIdx.x == 0) {
        // wavefronts that a role does not use end here (a barrier waits only for those that have not ended)
        if (threadIdx.x >= KVQ_STEP_K_NT) return;
        const StepFrontArgs a = *pa;
        k_quant_token<BITS, KVQ_STEP_K_NT>(a.params, a.D, a.cap, a.n, a.k_new, a.k_codes, a.k_ptr, a.ksp, a.cap_nnz_k, 1,
                                           a.d_status, 0);
        qk_sparse_new_token<R>(a);
    } else if (blockIdx.x == 1) {
        if (threadIdx.x >= 64 * W) return;
        const StepFrontArgs a = *pa;
        v_quant_token4<BITS, 4, W>(a.params, a.D, a.cap, a.n, a.k_side, a.v_new, a.v_codes, a.v_sz, a.v_ptr, a.vsp,
                                   a.cap_nnz_v, a.d_status, 0);
    } else {
        const KvqSparseFlat ksp{pa->ksp.idx, pa->ksp.val};
        qk_sparse_body<R, 8, KvqSparseFlat>((int)blockIdx.x - 2, pa->params, pa->D, pa->n_q_heads, pa->n, pa->k_ptr, ksp,
                                            (uint32_t)pa->cap_nnz_k, pa->q_rot, pa->scale, pa->scores, pa->ld,
                                            pa->tokens_per_wave);
    }
#endif
}

}  // namespace

// The first n_sink tokens are also kept as they came (paper Sec. 3.5): copy their rows.
static kvq_status copy_sink_rows(const kvq_cache *cache, uint16_t *sink, const uint16_t *src, int64_t n0, int32_t T,
                                 hipStream_t s)
{
    if (n0 >= cache->n_sink) return KVQ_OK;
    const int64_t rows = (cache->n_sink - n0 < T) ? cache->n_sink - n0 : T;
    const size_t D = (size_t)cache->n_kv_heads * KVQ_HEAD_DIM;
    KVQ_HIP_CHECK(hipMemcpyAsync(sink + n0 * D, src, (size_t)rows * D * 2, hipMemcpyDeviceToDevice, s));
    return KVQ_OK;
}

// Workgroup width of the quantization kernels.  A token's workgroup spends most of its time between
// barriers; 1024 threads finish a token soonest (what a decode step needs), while 256-thread
// workgroups, four to a compute unit and out of step with each other, get more tokens per second out
// of a bulk append.
static bool wide_wg(int D, int T) { return D >= 2048 && T < KVQ_BULK_TOKENS; }

static kvq_status append_checks(const kvq_cache *cache, const void *src, int32_t T, int64_t n_now)
{
    kvq_status st = kvq_check_cache(cache);
    if (st != KVQ_OK) return st;
    if (!cache->loaded) return KVQ_ERR_NOT_LOADED;
    if (!src || ((uintptr_t)src & 1) || T < 1 || T > KVQ_MAX_APPEND) return KVQ_ERR_INVALID_ARG;
    if (n_now + T > cache->cap_tokens) return KVQ_ERR_CAPACITY;
    return KVQ_OK;
}

extern "C" kvq_status kvq_quantize_append_k(kvq_cache *cache, const uint16_t *d_k_new, int32_t T, void *stream)
{
    kvq_status st = append_checks(cache, d_k_new, T, cache ? cache->n_tokens_k : 0);
    if (st != KVQ_OK) return st;
    const int D = cache->n_kv_heads * KVQ_HEAD_DIM;
    hipStream_t s = (hipStream_t)stream;
    const int single = (T == 1);
    if (!single) {
        if (!cache->workspace || cache->workspace_bytes < (int64_t)T * 4) return KVQ_ERR_CAPACITY;
        uint32_t *cnt = (uint32_t *)cache->workspace;
        kvq_k_count<<<(T + KVQ_COUNT_NT / 64 - 1) / (KVQ_COUNT_NT / 64), KVQ_COUNT_NT, 0, s>>>(cache->params, D, T, d_k_new, cnt);
        kvq_ptr_scan<<<1, 1024, 0, s>>>(cache->k_ptr, cache->n_tokens_k, T, cnt, cache->cap_nnz_k, cache->d_status);
    }
#define LAUNCH_K(B)                                                                                             \
    do {                                                                                                        \
        if (T >= KVQ_WAVE_TOKENS)                                                                               \
            kvq_k_quant_wave<B><<<(T + KVQ_KW_NT / 64 - 1) / (KVQ_KW_NT / 64), KVQ_KW_NT, 0, s>>>(               \
                cache->params, D, T, cache->cap_tokens, cache->n_tokens_k, d_k_new, cache->k_codes,              \
                cache->k_ptr, ksp, cache->cap_nnz_k, cache->d_status);                                           \
        else if (wide_wg(D, T))                                                                                 \
            kvq_k_quant<B, 1024><<<T, 1024, 0, s>>>(cache->params, D, cache->cap_tokens, cache->n_tokens_k,      \
                                                    d_k_new, cache->k_codes, cache->k_ptr, ksp, cache->cap_nnz_k,    \
                                                    single, cache->d_status);                                    \
        else                                                                                                    \
            kvq_k_quant<B, 256><<<T, 256, 0, s>>>(cache->params, D, cache->cap_tokens, cache->n_tokens_k,        \
                                                  d_k_new, cache->k_codes, cache->k_ptr, ksp, cache->cap_nnz_k,      \
                                                  single, cache->d_status);                                      \
    } while (0)
    // one set of kernels per layout of the outlier entries (flat arrays or a list of blocks)
    const auto launch = [&](const auto ksp) {
        if (cache->bits == 2) LAUNCH_K(2);
        else if (cache->bits == 3) LAUNCH_K(3);
        else LAUNCH_K(4);
    };
    if (cache->nnz_block_shift) launch(kvq_blocked_k(cache));
    else launch(kvq_flat_k(cache));
#undef LAUNCH_K
    KVQ_HIP_CHECK(hipGetLastError());
    st = copy_sink_rows(cache, cache->sink_k, d_k_new, cache->n_tokens_k, T, s);
    if (st != KVQ_OK) return st;
    cache->n_tokens_k += T;
    return KVQ_OK;
}

extern "C" kvq_status kvq_quantize_append_v(kvq_cache *cache, const uint16_t *d_v_new, int32_t T, void *stream)
{
    kvq_status st = append_checks(cache, d_v_new, T, cache ? cache->n_tokens_v : 0);
    if (st != KVQ_OK) return st;
    const int D = cache->n_kv_heads * KVQ_HEAD_DIM;
    if (cache->k_side_v < 0 || 2 * (int64_t)cache->k_side_v >= D) return KVQ_ERR_INVALID_ARG;
    if (D > 16384) return KVQ_ERR_UNSUPPORTED;       // the per-token selection keeps the vector in LDS
    hipStream_t s = (hipStream_t)stream;
    const size_t dyn = 3 * (size_t)D;
#define LAUNCH_V4W(B, J, WV)                                                                                   \
    kvq_v_quant4<B, J, WV><<<T, 64 * (WV), 0, s>>>(cache->params, D, cache->cap_tokens, cache->n_tokens_v,     \
                                               cache->k_side_v, d_v_new, cache->v_codes, cache->v_sz,          \
                                               cache->v_ptr, vsp, cache->cap_nnz_v,                           \
                                               cache->d_status)
#define LAUNCH_V4(B, J) LAUNCH_V4W(B, J, KVQ_VW_WAVES)
#define LAUNCH_V(B)                                                                                             \
    do {                                                                                                        \
        if (D == 4096 && T < KVQ_VW_SMALL_TOKENS) LAUNCH_V4W(B, 4, 16);                                         \
        else if (D == 2048 && T < KVQ_VW_SMALL_TOKENS) LAUNCH_V4W(B, 4, 8);                                     \
        else if (D == 4096) LAUNCH_V4(B, 16);                                                                   \
        else if (D == 2048) LAUNCH_V4(B, 8);                                                                    \
        else if (D == 1024) LAUNCH_V4(B, 4);                                                                    \
        else if (D == 5120 && T >= KVQ_BULK_TOKENS) LAUNCH_V4(B, 20);                                           \
        else if (D == 6656 && T >= KVQ_BULK_TOKENS) LAUNCH_V4(B, 26);                                           \
        else if (D == 8192 && T >= KVQ_BULK_TOKENS) LAUNCH_V4(B, 32);                                           \
        else if (wide_wg(D, T))                                                                                 \
            kvq_v_quant<B, 1024><<<T, 1024, dyn, s>>>(cache->params, D, cache->cap_tokens, cache->n_tokens_v,    \
                                                      cache->k_side_v, d_v_new, cache->v_codes, cache->v_sz,     \
                                                      cache->v_ptr, vsp,                                         \
                                                      cache->cap_nnz_v, cache->d_status);                        \
        else                                                                                                    \
            kvq_v_quant<B, 256><<<T, 256, dyn, s>>>(cache->params, D, cache->cap_tokens, cache->n_tokens_v,      \
                                                    cache->k_side_v, d_v_new, cache->v_codes, cache->v_sz,       \
                                                    cache->v_ptr, vsp, cache->cap_nnz_v,                        \
                                                    cache->d_status);                                            \
    } while (0)
    const auto launch = [&](const auto vsp) {
        if (cache->bits == 2) LAUNCH_V(2);
        else if (cache->bits == 3) LAUNCH_V(3);
        else LAUNCH_V(4);
    };
    if (cache->nnz_block_shift) launch(kvq_blocked_v(cache));
    else launch(kvq_flat_v(cache));
#undef LAUNCH_V
#undef LAUNCH_V4
#undef LAUNCH_V4W
    KVQ_HIP_CHECK(hipGetLastError());
    st = copy_sink_rows(cache, cache->sink_v, d_v_new, cache->n_tokens_v, T, s);
    if (st != KVQ_OK) return st;
    cache->n_tokens_v += T;
    return KVQ_OK;
}

extern "C" kvq_status kvq_quantize_append_kv(kvq_cache *cache, const uint16_t *d_k_new, const uint16_t *d_v_new,
                                             int32_t T, void *stream)
{
    kvq_status st = append_checks(cache, d_k_new, T, cache ? cache->n_tokens_k : 0);
    if (st != KVQ_OK) return st;
    st = append_checks(cache, d_v_new, T, cache->n_tokens_v);
    if (st != KVQ_OK) return st;
    const int D = cache->n_kv_heads * KVQ_HEAD_DIM;
    if (cache->k_side_v < 0 || 2 * (int64_t)cache->k_side_v >= D) return KVQ_ERR_INVALID_ARG;
    if (D > 16384) return KVQ_ERR_UNSUPPORTED;       // the per-token Value selection keeps the vector in LDS
    if (T >= KVQ_KV_SPLIT_TOKENS) {
        // Such an append fills the GPU with either kernel alone, and compute units that run both bodies
        // at once are slower than the two launches one after the other (measured: 50 us against 44 us
        // for 256 tokens of 4096 channels, 233 us against 188 us for 4096); every check of both calls
        // has passed above.
        if (!cache->workspace || cache->workspace_bytes < (int64_t)T * 4) return KVQ_ERR_CAPACITY;
        st = kvq_quantize_append_k(cache, d_k_new, T, stream);
        if (st != KVQ_OK) return st;
        return kvq_quantize_append_v(cache, d_v_new, T, stream);
    }
    hipStream_t s = (hipStream_t)stream;
    const int single = (T == 1);
    if (!single) {
        if (!cache->workspace || cache->workspace_bytes < (int64_t)T * 4) return KVQ_ERR_CAPACITY;
        uint32_t *cnt = (uint32_t *)cache->workspace;
        kvq_k_count<<<(T + KVQ_COUNT_NT / 64 - 1) / (KVQ_COUNT_NT / 64), KVQ_COUNT_NT, 0, s>>>(cache->params, D, T, d_k_new, cnt);
        kvq_ptr_scan<<<1, 1024, 0, s>>>(cache->k_ptr, cache->n_tokens_k, T, cnt, cache->cap_nnz_k, cache->d_status);
    }
    const size_t dyn = 3 * (size_t)D;
#define LAUNCH_KV(B)                                                                     \
    do {                                                                                 \
        if (wide_wg(D, T)) kvq_kv_quant<B, 1024><<<2 * T, 1024, dyn, s>>>(a);            \
        else kvq_kv_quant<B, 256><<<2 * T, 256, dyn, s>>>(a);                            \
    } while (0)
    const auto launch = [&](const auto ksp, const auto vsp) {
        KvAppendArgs<std::remove_cv_t<decltype(ksp)>> a;
        a.params = cache->params; a.D = D; a.k_side = cache->k_side_v; a.single = single;
        a.cap = cache->cap_tokens; a.n0_k = cache->n_tokens_k; a.n0_v = cache->n_tokens_v;
        a.cap_nnz_k = cache->cap_nnz_k; a.cap_nnz_v = cache->cap_nnz_v;
        a.k_new = d_k_new; a.v_new = d_v_new;
        a.k_codes = cache->k_codes; a.v_codes = cache->v_codes; a.v_sz = cache->v_sz;
        a.k_ptr = cache->k_ptr; a.v_ptr = cache->v_ptr;
        a.ksp = ksp; a.vsp = vsp;
        a.d_status = cache->d_status;
        if (cache->bits == 2) LAUNCH_KV(2);
        else if (cache->bits == 3) LAUNCH_KV(3);
        else LAUNCH_KV(4);
    };
    if (cache->nnz_block_shift) launch(kvq_blocked_k(cache), kvq_blocked_v(cache));
    else launch(kvq_flat_k(cache), kvq_flat_v(cache));
#undef LAUNCH_KV
    KVQ_HIP_CHECK(hipGetLastError());
    st = copy_sink_rows(cache, cache->sink_k, d_k_new, cache->n_tokens_k, T, s);
    if (st != KVQ_OK) return st;
    st = copy_sink_rows(cache, cache->sink_v, d_v_new, cache->n_tokens_v, T, s);
    if (st != KVQ_OK) return st;
    cache->n_tokens_k += T;
    cache->n_tokens_v += T;
    return KVQ_OK;
}


template <int BITS, int R, int W>
static kvq_status step_front_launch_brw(kvq_cache *cache, StepFrontArgs &a, hipStream_t s, bool *done, bool dry)
{
    // static LDS of the kernel (the append bodies' arrays) comes on top of the sparse role's dynamic LDS
    static const int static_lds = [] {
        hipFuncAttributes fa;
        if (hipFuncGetAttributes(&fa, (const void *)kvq_step_front<BITS, R, W>) != hipSuccess) return -1;
        return (int)fa.sharedSizeBytes;
    }();
    static const hipError_t lds_attr = hipFuncSetAttribute((const void *)kvq_step_front<BITS, R, W>,
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 147456 - 16384);
    if (static_lds < 0 || static_lds > 16384) return KVQ_OK;             // *done stays false
    KVQ_HIP_CHECK(lds_attr);
    QkSparsePlan plan;
    if (!qk_sparse_plan(cache->n_q_heads, a.n, 8, (size_t)static_lds, plan) || plan.waves != 16) return KVQ_OK;
    if (plan.lds < (size_t)cache->n_q_heads * 8) return KVQ_OK;
    a.tokens_per_wave = plan.tokens_per_wave;
    if (dry) {                                    // the caller only asks whether this launch applies
        *done = true;
        return KVQ_OK;
    }
    kvq_status st = copy_sink_rows(cache, cache->sink_k, a.k_new, a.n, 1, s);
    if (st != KVQ_OK) return st;
    st = copy_sink_rows(cache, cache->sink_v, a.v_new, a.n, 1, s);
    if (st != KVQ_OK) return st;
    kvq_step_front<BITS, R, W><<<plan.grid + 2, 1024, plan.lds, s>>>(a);
    KVQ_HIP_CHECK(hipGetLastError());
    cache->n_tokens_k += 1;
    cache->n_tokens_v += 1;
    *done = true;
    return KVQ_OK;
}

template <int BITS, int R>
static kvq_status step_front_launch_br(kvq_cache *cache, StepFrontArgs &a, hipStream_t s, bool *done, bool dry)
{
    if (a.D == 4096) return step_front_launch_brw<BITS, R, 16>(cache, a, s, done, dry);
    return step_front_launch_brw<BITS, R, 4>(cache, a, s, done, dry);
}

template <int BITS>
static kvq_status step_front_launch_b(kvq_cache *cache, StepFrontArgs &a, hipStream_t s, bool *done, bool dry)
{
    switch (cache->n_q_heads / cache->n_kv_heads) {
    case 1: return step_front_launch_br<BITS, 1>(cache, a, s, done, dry);
    case 2: return step_front_launch_br<BITS, 2>(cache, a, s, done, dry);
    case 4: return step_front_launch_br<BITS, 4>(cache, a, s, done, dry);
    case 8: return step_front_launch_br<BITS, 8>(cache, a, s, done, dry);
    default: return KVQ_OK;
    }
}

static kvq_status step_front(kvq_cache *cache, const uint16_t *d_k_new, const uint16_t *d_v_new,
                             const float *d_q_rot, float scale, float *d_scores, int64_t ld_scores, hipStream_t s,
                             bool *done, bool dry)
{
    *done = false;
    kvq_status st = append_checks(cache, d_k_new, 1, cache ? cache->n_tokens_k : 0);
    if (st != KVQ_OK) return st;
    st = append_checks(cache, d_v_new, 1, cache->n_tokens_v);
    if (st != KVQ_OK) return st;
    const int D = cache->n_kv_heads * KVQ_HEAD_DIM;
    if (cache->k_side_v < 0 || 2 * (int64_t)cache->k_side_v >= D) return KVQ_ERR_INVALID_ARG;
    // shapes this launch covers; every other one takes the two calls
    if (D != 1024 && D != 4096) return KVQ_OK;
    if (cache->nnz_block_shift || (cache->loaded & 2) || cache->n_tokens_k != cache->n_tokens_v) return KVQ_OK;
    if (cache->cap_nnz_k >= ((int64_t)1 << 31)) return KVQ_OK;
    const int64_t per_token = cache->cap_nnz_k / (cache->cap_tokens > 0 ? cache->cap_tokens : 1);
    if (per_token < 16 && cache->n_q_heads <= 32) return KVQ_OK;         // the sparse kernel would take 32-token sub-ranges
    StepFrontArgs a;
    a.params = cache->params; a.D = D; a.n_q_heads = cache->n_q_heads; a.k_side = cache->k_side_v;
    a.cap = cache->cap_tokens; a.n = cache->n_tokens_k;
    a.cap_nnz_k = cache->cap_nnz_k; a.cap_nnz_v = cache->cap_nnz_v;
    a.k_new = d_k_new; a.v_new = d_v_new;
    a.k_codes = cache->k_codes; a.v_codes = cache->v_codes; a.v_sz = cache->v_sz;
    a.k_ptr = cache->k_ptr; a.v_ptr = cache->v_ptr;
    a.ksp = kvq_flat_k(cache); a.vsp = kvq_flat_v(cache);
    a.d_status = cache->d_status;
    a.q_rot = d_q_rot; a.scale = scale; a.scores = d_scores; a.ld = ld_scores; a.tokens_per_wave = 1;
    if (cache->bits == 2) return step_front_launch_b<2>(cache, a, s, done, dry);
    if (cache->bits == 3) return step_front_launch_b<3>(cache, a, s, done, dry);
    return step_front_launch_b<4>(cache, a, s, done, dry);
}

kvq_status kvq_step_front_launch(kvq_cache *cache, const uint16_t *d_k_new, const uint16_t *d_v_new,
                                 const float *d_q_rot, float scale, float *d_scores, int64_t ld_scores, hipStream_t s,
                                 bool *done)
{
    return step_front(cache, d_k_new, d_v_new, d_q_rot, scale, d_scores, ld_scores, s, done, false);
}

extern "C" int32_t kvq_decode_step_launches(const kvq_cache *cache)
{
    if (!cache) return -1;
    kvq_cache view = *cache;                     // a dry run: nothing is launched, nothing advances
    bool front = false;
    static const uint16_t dummy[2] = {0, 0};     // the checks only look at alignment
    if (step_front(&view, dummy, dummy, nullptr, 0.f, nullptr, 0, nullptr, &front, true) != KVQ_OK) return -1;
    const int sink = cache->n_sink > 0 ? 1 : 0;
    // the two calls: append, sparse Key (unless the thresholds admit no outlier), dense Key, sparse Value,
    // dense Value, reduction
    const int two_calls = (cache->loaded & 2) ? 5 : 6;
    return (front ? 5 : two_calls) + sink;
}

extern "C" kvq_status kvq_calibrate_key_channels(const uint16_t *d_k_cal, int32_t T, int32_t D, float outlier_fraction,
                                                 uint16_t *d_s, uint16_t *d_z, uint16_t *d_lo, uint16_t *d_hi,
                                                 void *stream)
{
    if (!d_k_cal || !d_s || !d_z || !d_lo || !d_hi || ((uintptr_t)d_k_cal & 1)) return KVQ_ERR_INVALID_ARG;
    if (T < 1 || D < 1 || !(outlier_fraction >= 0.0f) || !(outlier_fraction < 1.0f)) return KVQ_ERR_INVALID_ARG;
    if (T > 32768) return KVQ_ERR_UNSUPPORTED;        // a channel's calibration values are kept in LDS
    const int k = (int)floorf(outlier_fraction * 0.5f * (float)T + 0.5f);
    if (2 * k >= T) return KVQ_ERR_INVALID_ARG;
    const size_t dyn = 3 * (size_t)T;
    static size_t lds_attr = 0;
    if (dyn > lds_attr) {
        KVQ_HIP_CHECK(hipFuncSetAttribute((const void *)kvq_calib_channel<1024>,
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn));
        lds_attr = dyn;
    }
    kvq_calib_channel<1024><<<D, 1024, dyn, (hipStream_t)stream>>>(d_k_cal, T, D, k, d_s, d_z, d_lo, d_hi);
    KVQ_HIP_CHECK(hipGetLastError());
    return KVQ_OK;
}
