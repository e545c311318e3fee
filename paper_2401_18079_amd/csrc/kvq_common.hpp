// Shared declarations of the kvq HIP library (gfx950 only): parameter-block layout, storage-format
// addressing, small device helpers.  Nothing in this file is shared with the CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/kvq.h"

#define KVQ_HEAD_DIM 128
#define KVQ_MAX_APPEND 4096
#define KVQ_NOALLOC_MAX_Q_HEADS 32

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

// ---- device parameter block written by kvq_lut_load --------------------------------------
// Fixed header followed by per-channel arrays of D entries each.
struct KvqParamsHeader {
    float lut_k[16];      // sorted signposts, Keys
    float lut_v[16];      // sorted signposts, Values
    float rope_vh[64];    // theta_i / (2 pi), fp32 head of a two-term split
    float rope_vl[64];    // fp32 tail: (theta_i / (2 pi)) - rope_vh[i]
    int32_t D;
    int32_t bits;
    int32_t pad[30];
    float rope_cd[64];    // cos(KVQ_ROPE_STEP * theta_i): the rotation that advances a token's (cos, sin)
    float rope_sd[64];    // sin(KVQ_ROPE_STEP * theta_i)   of pair i by KVQ_ROPE_STEP positions
};
constexpr int KVQ_ROPE_STEP = 1024;
constexpr int KVQ_PARAMS_HEADER_BYTES = 1280;
static_assert(sizeof(KvqParamsHeader) == KVQ_PARAMS_HEADER_BYTES, "header layout");

struct KvqParamsView {          // device pointers into the block
    const KvqParamsHeader *hdr;
    const uint16_t *s16, *z16, *lo16, *hi16;   // raw fp16 inputs [D]
    const float *s, *z, *rinv, *lo, *hi;       // fp32 expansions [D]; rinv = 1.0f / s (IEEE)
};

__host__ __device__ inline int64_t kvq_params_bytes_D(int D) { return KVQ_PARAMS_HEADER_BYTES + (int64_t)D * (4 * 2 + 5 * 4); }

__host__ __device__ inline KvqParamsView kvq_params_view(const void *block, int D)
{
    KvqParamsView v;
    const char *p = (const char *)block;
    v.hdr = (const KvqParamsHeader *)p;
    p += KVQ_PARAMS_HEADER_BYTES;
    v.s16 = (const uint16_t *)p; p += 2 * (int64_t)D;
    v.z16 = (const uint16_t *)p; p += 2 * (int64_t)D;
    v.lo16 = (const uint16_t *)p; p += 2 * (int64_t)D;
    v.hi16 = (const uint16_t *)p; p += 2 * (int64_t)D;
    v.s = (const float *)p; p += 4 * (int64_t)D;
    v.z = (const float *)p; p += 4 * (int64_t)D;
    v.rinv = (const float *)p; p += 4 * (int64_t)D;
    v.lo = (const float *)p; p += 4 * (int64_t)D;
    v.hi = (const float *)p;
    return v;
}

// 16-byte load of data that is read once per launch (packed codes): the non-temporal hint keeps the
// stream from displacing what is read again (scores, partial sums) and a plain read of a large
// buffer is measurably faster with it.
__device__ __forceinline__ uint4 kvq_load_stream16(const void *p)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = __builtin_nontemporal_load((const u32x4 *)p);
    return uint4{v.x, v.y, v.z, v.w};
}

// ---- storage format addressing (bytes) -----------------------------------------------------
// Key chunk of (token n, KV head h): `bits` pieces of 16 bytes, piece j at k_piece0 + j*1024.
__host__ __device__ inline int64_t kvq_k_piece0(int bits, int64_t cap, int64_t n, int h)
{
    return (int64_t)h * cap * 16 * bits + (n >> 6) * (64 * 16 * bits) + (n & 63) * 16;
}
// Value chunk of (token pair m, KV head h, channel half g).
__host__ __device__ inline int64_t kvq_v_piece0(int bits, int64_t cap, int64_t m, int h, int g)
{
    return (int64_t)(h * 2 + g) * (cap >> 1) * 16 * bits + (m >> 6) * (64 * 16 * bits) + (m & 63) * 16;
}

// ---- small device helpers -------------------------------------------------------------------
__device__ inline float kvq_h2f(uint16_t b) { return (float)__builtin_bit_cast(half_t, b); }
__device__ inline uint16_t kvq_f2h_rn(float f) { return __builtin_bit_cast(uint16_t, (half_t)f); }

// Nearest signpost by exhaustive search in fp32, ties to the smaller index.  Also returns the
// signpost itself so callers need no dynamically indexed register array.
template <int NE>
__device__ inline int kvq_nearest(const float *lut, float xn, float &signpost)
{
    int best = 0;
    float bestd = __builtin_fabsf(xn - lut[0]);
    float bestv = lut[0];
#pragma unroll
    for (int j = 1; j < NE; ++j) {
        float dj = __builtin_fabsf(xn - lut[j]);
        if (dj < bestd) { bestd = dj; best = j; bestv = lut[j]; }
    }
    signpost = bestv;
    return best;
}

// (x & mask) | bits in one instruction (the compiler emits an AND and an OR/ADD for this pattern).
// The mask travels in a scalar register: VOP3 instructions take no 32-bit literals on gfx9.
__device__ __forceinline__ uint32_t kvq_and_or(uint32_t x, uint32_t mask, uint32_t bits)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(mask), "v"(bits));
    return r;
}

// Scatter-add of floats into LDS without floating-point atomics (ds_add_f32 processes lanes one at a
// time on gfx950, roughly 30x slower than integer LDS atomics): the value is converted to 64-bit
// fixed point and added with an integer atomic.  Integer addition is associative, so the result does
// not depend on the order in which lanes arrive.
//
// kvq_to_fixed<SH>(x) = x * 2^(32+SH) as a two's-complement 64-bit integer, for |x| < 2^(31-SH):
// integer part (floor) in the high word, fraction in the low word.  Non-negative values are exact
// down to 2^-(32+SH); the fraction of a negative value (1 - frac|y|) is rounded to fp32, an absolute
// error of at most 2^-(24+SH) per value.
template <int SH>
__device__ __forceinline__ unsigned long long kvq_to_fixed(float x)
{
    const float y = x * (float)(1 << SH);
    const int hi = (int)__builtin_floorf(y);
    const uint32_t lo = (uint32_t)(__builtin_amdgcn_fractf(y) * 4294967296.0f);
    return ((unsigned long long)(uint32_t)hi << 32) | lo;
}
template <int SH>
__device__ __forceinline__ float kvq_from_fixed(unsigned long long v)
{
    const long long sv = (long long)v;
    const unsigned long long m = (unsigned long long)(sv < 0 ? -sv : sv);    // magnitude: no cancellation below
    const float r = ((float)(uint32_t)(m >> 32) + (float)(uint32_t)m * (1.0f / 4294967296.0f)) * (1.0f / (float)(1 << SH));
    return sv < 0 ? -r : r;
}
// Same conversion in three instructions; the low word is rounded to fp32 before the (possibly
// cancelling) addition, an absolute error of at most 2^-(25+SH).
template <int SH>
__device__ __forceinline__ float kvq_from_fixed_fast(unsigned long long v)
{
    const float hi = (float)(int)(uint32_t)(v >> 32), lo = (float)(uint32_t)v;
    return __builtin_fmaf(lo, 1.0f / 4294967296.0f, hi) * (1.0f / (float)(1 << SH));
}
template <int SH>
__device__ __forceinline__ void kvq_lds_add_fixed(unsigned long long *cell, float x)
{
    atomicAdd(cell, kvq_to_fixed<SH>(x));
}

// ---- helpers shared by the two balanced sparse kernels (lanes = outlier entries) ----------------

// Where the (channel index, residual) entries of one side of the cache live: two flat arrays, or
// lists of blocks (paper App. "Limitations": the outlier storage allocated in blocks, so that an
// append never copies what is stored).  The kernels that touch the entries are templates over the
// two, so the flat layout pays nothing for the other.
struct KvqSparseFlat {
    uint16_t *idx, *val;
    __device__ __forceinline__ void put(uint64_t e, uint16_t i, uint16_t v) const
    {
        idx[e] = i;
        val[e] = v;
    }
};
// Entry e is element e & (2^shift - 1) of block e >> shift; idx_b / val_b are device arrays of device
// pointers, one per block, every slot below the capacity valid.
struct KvqSparseBlocked {
    uint16_t *const *idx_b, *const *val_b;
    int shift;
    __device__ __forceinline__ void put(uint64_t e, uint16_t i, uint16_t v) const
    {
        const uint64_t b = e >> shift, o = e & ((1ull << shift) - 1);
        idx_b[b][o] = i;
        val_b[b][o] = v;
    }
};

// One batch of U x 64 index/value loads starting at entry `eb` (lane l takes entries eb + l + 64 u).
// CLAMP = false: the whole batch lies inside the arrays (possibly past the sub-range's end `e_end`,
// where the loaded values are ignored), one address per lane plus immediate offsets; CLAMP = true:
// lanes past the end re-read the last entry.  Groups of 64 entries that lie entirely past `e_end`
// are skipped (a wavefront-uniform branch).  `nnz_cap` is the capacity in entries.
template <bool CLAMP, int U>
__device__ __forceinline__ void kvq_sparse_load_batch(const KvqSparseFlat &sp, uint32_t /*nnz_cap*/, uint32_t eb,
                                                      uint32_t e_end, int lane, uint32_t (&chv)[U],
                                                      uint32_t (&vb)[U])
{
    const char *__restrict__ ib = (const char *)sp.idx;
    const char *__restrict__ vbp = (const char *)sp.val;
    if (!CLAMP) {
        const uint32_t off0 = (eb + (uint32_t)lane) * 2u;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (eb + 64u * u >= e_end) break;            // uniform: the rest of the batch is past the end
            chv[u] = *(const uint16_t *)(ib + (size_t)off0 + 128 * u);
            vb[u] = *(const uint16_t *)(vbp + (size_t)off0 + 128 * u);
        }
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (eb + 64u * u >= e_end) break;
            uint32_t e = eb + (uint32_t)lane + 64u * u;
            e = (e < e_end) ? e : e_end - 1;
            chv[u] = *(const uint16_t *)(ib + (size_t)(e * 2u));
            vb[u] = *(const uint16_t *)(vbp + (size_t)(e * 2u));
        }
    }
}

// Blocked storage: a block holds at least 1024 entries and a batch fewer, so a batch touches the
// block of its first entry and at most the one after; `eb` is wavefront-uniform, which makes the
// block pointers scalar loads.
template <bool CLAMP, int U>
__device__ __forceinline__ void kvq_sparse_load_batch(const KvqSparseBlocked &sp, uint32_t nnz_cap, uint32_t eb,
                                                      uint32_t e_end, int lane, uint32_t (&chv)[U],
                                                      uint32_t (&vb)[U])
{
    static_assert(64 * U <= (1 << KVQ_NNZ_BLOCK_SHIFT_MIN), "a batch must fit in the smallest block");
    const uint32_t sh = (uint32_t)sp.shift, mask = (1u << sh) - 1u;
    const uint32_t b0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)(eb >> sh));
    const uint32_t n_blocks = nnz_cap >> sh;
    const uint32_t b1 = (b0 + 1u < n_blocks) ? b0 + 1u : b0;
    const uint16_t *i0 = sp.idx_b[b0], *v0 = sp.val_b[b0];
    const uint16_t *i1 = sp.idx_b[b1], *v1 = sp.val_b[b1];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (eb + 64u * u >= e_end) break;
        uint32_t e = eb + (uint32_t)lane + 64u * u;
        if (CLAMP) e = (e < e_end) ? e : e_end - 1;
        const bool first = (e >> sh) == b0;
        const uint32_t o = e & mask;
        chv[u] = (first ? i0 : i1)[o];
        vb[u] = (first ? v0 : v1)[o];
    }
}

// Token (relative to the sub-range) of entry `e` = `first` + lane.  `pw` holds the sub-range's
// pointers (lane j: first entry of token j; lanes >= tc: the end), `tcur` is the wavefront's cursor:
// the token that entry `first` belongs to once advanced.  Everything but the final compare-and-add
// is scalar work on values read out of `pw` with v_readlane.
__device__ __forceinline__ int kvq_sparse_token(uint32_t pw, int tc, int &tcur, uint32_t first, uint32_t e)
{
    while (tcur + 1 < tc && (uint32_t)__builtin_amdgcn_readlane((int)pw, tcur + 1) <= first) ++tcur;
    int t = tcur;
    int j = tcur + 1;
    while (j < tc) {
        const uint32_t pj = (uint32_t)__builtin_amdgcn_readlane((int)pw, j);
        if (pj > first + 63u) break;
        t += (e >= pj) ? 1 : 0;
        j = __builtin_amdgcn_readfirstlane(j + 1);       // keeps the loop counter in a scalar register
    }
    return t;
}

// The same without a loop, for sub-ranges of many short tokens (where kvq_sparse_token walks a dozen
// pointers per group of 64 entries, in scalar code that nothing overlaps): the token of entry
// first + lane is the largest j with pw_j <= first + lane.  Pointer lane j (1 <= j < tc) whose token
// starts at or before entry first + 63 leaves j in slot max(pw_j - first, 0) of `slots` (64 words of
// LDS private to the wavefront; equal pointers, i.e. empty tokens, meet in one slot: an atomic
// maximum); an entry's token is the running maximum of the slots up to its own, a prefix scan over
// the lanes with DPP moves.  All 64 lanes must be active.
__device__ __forceinline__ uint32_t kvq_dpp_max_u32(uint32_t v, uint32_t moved)
{
    return v > moved ? v : moved;
}
__device__ __forceinline__ int kvq_sparse_token_scan(uint32_t pw, int tc, uint32_t first, int lane, uint32_t *slots)
{
    slots[lane] = 0u;
    const bool before = pw <= first;
    const uint32_t rel = before ? 0u : pw - first;
    if (lane >= 1 && lane < tc && rel <= 63u)
        __hip_atomic_fetch_max(&slots[rel], (uint32_t)lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    uint32_t v = slots[lane];
    // inclusive prefix maximum: inside each row of 16 lanes (a lane without a source keeps 0), then
    // lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into rows 2 and 3
    v = kvq_dpp_max_u32(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false));
    v = kvq_dpp_max_u32(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false));
    v = kvq_dpp_max_u32(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false));
    v = kvq_dpp_max_u32(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false));
    v = kvq_dpp_max_u32(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false));
    v = kvq_dpp_max_u32(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false));
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");          // the next group clears the slots
    __builtin_amdgcn_wave_barrier();
    return (int)v;
}

// Issue priority of the calling wavefront, 0 (lowest) to 3.  The SIMD's arbiter serves the highest
// priority first and, among equals, the OLDEST wavefront: the four wavefronts that share a SIMD for a
// whole kernel then finish one after the other (measured on the dense Value kernel: workgroups
// dispatched first end at 34 us, those dispatched last at 48 us, and the tail runs with the SIMDs a
// quarter full).  A wavefront that calls this with (its slot on the SIMD + a step counter) & 3 at every
// step spends a quarter of its steps at each priority, so the four advance at the same average rate.
// The instruction takes an immediate operand, hence the switch.
__device__ __forceinline__ void kvq_set_wave_priority(int p)
{
    // `p` must be wavefront-uniform; the read below also tells the compiler so (a divergent switch
    // would run every case, one after the other, under execution masks)
    switch (__builtin_amdgcn_readfirstlane(p) & 3) {
    case 0: __builtin_amdgcn_s_setprio(0); break;
    case 1: __builtin_amdgcn_s_setprio(1); break;
    case 2: __builtin_amdgcn_s_setprio(2); break;
    default: __builtin_amdgcn_s_setprio(3); break;
    }
}

// ---- softmax hand-over from the Key kernels to the Value kernels (fused decode call) ------------
// The Key kernels leave the maximum of the scores they wrote in per-head slots: a head owns
// KVQ_STAT_SLOTS consecutive floats, one per workgroup of the dense Key kernel that covers the head
// (at most 256) plus one per attention-sink token.  A Value kernel takes the maximum m over a head's
// slots and weights token n by e_n = 2^(log2(e) (x_n - m)) = exp(x_n - m); the sum of the e_n is
// gathered along the way and the final reduction divides by it.
constexpr int KVQ_STAT_SLOTS = 256 + KVQ_MAX_SINK;
constexpr float KVQ_LOG2E = 1.44269504088896340736f;
constexpr float KVQ_STAT_FLOOR = -3.0e38f;      // "no score": finite, so that differences stay finite

// v of the lane `N` places to the right inside the lane's row of 16 (rotating): a DPP operand
// modifier, no LDS traffic and a few cycles of latency (a cross-lane shuffle costs a hundred).
template <int N>
__device__ __forceinline__ float kvq_row_ror(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x120 + N, 0xf, 0xf, false));
}
__device__ __forceinline__ float kvq_wave_max(float v)        // maximum over the 64 lanes, in every lane
{
    v = __builtin_fmaxf(v, kvq_row_ror<8>(v));                // every lane ends up with its row's maximum
    v = __builtin_fmaxf(v, kvq_row_ror<4>(v));
    v = __builtin_fmaxf(v, kvq_row_ror<2>(v));
    v = __builtin_fmaxf(v, kvq_row_ror<1>(v));
    const int b = __builtin_bit_cast(int, v);                 // the four rows' maxima as scalars
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return __builtin_fmaxf(__builtin_fmaxf(r0, r1), __builtin_fmaxf(r2, r3));
}
// Unnormalised softmax weight of score x given m2 = log2(e) * (maximum score of the head).
__device__ __forceinline__ float kvq_stat_weight(float x, float m2)
{
    return __builtin_amdgcn_exp2f(x * KVQ_LOG2E - m2);
}

// The two halves of the fused decode call (kvq_attention_decode), defined beside the kernels they
// launch.  kvq_qk_run: as kvq_qk_matvec; with `stat_slots` non-null the kernels also fill the slots
// and *n_stat receives how many of each head's slots are in use.  kvq_pv_run: as kvq_pv_matvec; with
// `stat_slots` non-null `weights` holds raw scores and the result is the softmax-weighted sum.
__attribute__((visibility("hidden"))) kvq_status kvq_qk_run(const kvq_cache *cache, const float *d_q_rot, float scale,
                                                            float *d_scores, int64_t ld, float *stat_slots,
                                                            int *n_stat, hipStream_t s);
__attribute__((visibility("hidden"))) kvq_status kvq_pv_run(const kvq_cache *cache, const float *d_weights, int64_t ld,
                                                            float *d_out, const float *stat_slots, int n_stat,
                                                            hipStream_t s);
// kvq_cache.loaded: bit 0 set by kvq_lut_load, bit 1 by it too when the thresholds admit no Key outlier.
// Bit 2 never appears in a caller's descriptor: kvq_decode_step sets it on its own copy when its first
// launch has already written the sparse part of the scores.
#define KVQ_LOADED_SPARSE_SCORES_DONE 4
// First launch of kvq_decode_step: the append of one token's Key and Value and the sparse Key kernel over
// the tokens before it, as workgroups of one kernel (kvq_append.hip).  *done = false, nothing launched,
// nothing changed: the shape is not covered and the caller takes the two calls instead.
__attribute__((visibility("hidden"))) kvq_status kvq_step_front_launch(kvq_cache *cache, const uint16_t *d_k_new,
                                                                       const uint16_t *d_v_new, const float *d_q_rot,
                                                                       float scale, float *d_scores, int64_t ld_scores,
                                                                       hipStream_t s, bool *done);
// Bytes of the workspace that kvq_pv_run uses (from its start); the statistics slots follow.
__attribute__((visibility("hidden"))) int64_t kvq_pv_workspace_bytes(int n_q_heads);

// Optional per-kernel timing (kvq_profile_enable) of the dense kernels, two ways.  (1) A ring of HIP
// event pairs recorded around the launch: what the stream sees between the end of the kernel before
// and the end of this one (the records themselves stall the queue by a few microseconds each).
// (2) The kernel's own span: the first thread of every workgroup stores the GPU's constant-rate wall
// clock when the workgroup starts and, after a barrier at the very end, when all its wavefronts are
// done (plain stores to the workgroup's own slot of a caller-provided device buffer: atomics on one
// address would stall the kernel they are meant to time).  First start to last end over the
// workgroups is the span a kernel trace reports, and nothing is inserted between kernels.
// Buffer layout: [2 kernels][RING calls][KVQ_PROFILE_MAX_WGS][start, end], 64-bit ticks, zero = unused.
constexpr int KVQ_PROFILE_RING = 256;
constexpr int KVQ_PROFILE_MAX_WGS = 1024;
struct KvqProfile {
    int enabled;
    hipEvent_t ev[2][KVQ_PROFILE_RING][2];     // [QK, PV][call % ring][start, stop]
    int64_t count[2];                          // calls recorded since the last enable
    unsigned long long *spans;                 // device buffer or null
    int use_events;                            // record the event pairs too
};
// The slots of the next call of kernel `which` (for a launch of n_wgs workgroups), or null when spans
// are not being taken or the launch has more workgroups than a call has slots.
inline unsigned long long *kvq_profile_span_slot(KvqProfile &p, int which, int64_t n_wgs)
{
    if (!p.enabled || !p.spans || n_wgs > KVQ_PROFILE_MAX_WGS) return nullptr;
    return p.spans + ((int64_t)which * KVQ_PROFILE_RING + (p.count[which] % KVQ_PROFILE_RING)) * KVQ_PROFILE_MAX_WGS * 2;
}
__device__ __forceinline__ void kvq_span_start(unsigned long long *slots)
{
    if (slots && threadIdx.x == 0)
        slots[2 * (blockIdx.y * gridDim.x + blockIdx.x)] = (unsigned long long)wall_clock64();
}
// Every thread of the workgroup must call this (it holds a barrier when spans are being taken).
__device__ __forceinline__ void kvq_span_end(unsigned long long *slots)
{
    if (slots) {
        // this wavefront's stores have been acknowledged (a wait only: a fence would also write back
        // and invalidate caches that the workgroups still running depend on)
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0)
            slots[2 * (blockIdx.y * gridDim.x + blockIdx.x) + 1] = (unsigned long long)wall_clock64();
    }
}
KvqProfile &kvq_profile_state();

// Compute units of the current device (MI355X: 256), asked once per process; launch plans size their
// grids from it.  A failed query falls back to 256.
inline int kvq_cu_count()
{
    static const int n = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return 256;
        return cus;
    }();
    return n;
}

#define KVQ_HIP_CHECK(expr)                         \
    do {                                            \
        hipError_t _e = (expr);                     \
        if (_e != hipSuccess) return KVQ_ERR_HIP;   \
    } while (0)

static inline kvq_status kvq_check_cache(const kvq_cache *c)
{
    if (!c) return KVQ_ERR_INVALID_ARG;
    if (c->bits < 2 || c->bits > 4 || c->head_dim != KVQ_HEAD_DIM) return KVQ_ERR_UNSUPPORTED;
    if (c->n_kv_heads < 1 || c->n_q_heads < c->n_kv_heads || c->n_q_heads % c->n_kv_heads) return KVQ_ERR_INVALID_ARG;
    if ((int64_t)c->n_kv_heads * KVQ_HEAD_DIM > 65536) return KVQ_ERR_UNSUPPORTED;
    if (c->cap_tokens <= 0 || (c->cap_tokens & 127) || c->cap_tokens >= ((int64_t)1 << 24)) return KVQ_ERR_INVALID_ARG;
    if (c->n_tokens_k < 0 || c->n_tokens_k > c->cap_tokens || c->n_tokens_v < 0 || c->n_tokens_v > c->cap_tokens)
        return KVQ_ERR_INVALID_ARG;
    const void *ptrs[] = {c->params, c->k_codes, c->v_codes, c->v_sz, c->k_ptr, c->v_ptr, c->d_status};
    for (const void *p : ptrs)
        if (!p || ((uintptr_t)p & 15)) return KVQ_ERR_INVALID_ARG;
    if (c->nnz_block_shift == 0) {
        const void *flat[] = {c->k_idx, c->k_val, c->v_idx, c->v_val};
        for (const void *p : flat)
            if (!p || ((uintptr_t)p & 15)) return KVQ_ERR_INVALID_ARG;
    } else {
        // blocked sparse arrays: 2^10 .. 2^30 entries per block, whole blocks, at least one
        if (c->nnz_block_shift < KVQ_NNZ_BLOCK_SHIFT_MIN || c->nnz_block_shift > KVQ_NNZ_BLOCK_SHIFT_MAX)
            return KVQ_ERR_INVALID_ARG;
        const int64_t be = (int64_t)1 << c->nnz_block_shift;
        if (c->cap_nnz_k < be || (c->cap_nnz_k & (be - 1)) || c->cap_nnz_v < be || (c->cap_nnz_v & (be - 1)))
            return KVQ_ERR_INVALID_ARG;
        const void *tabs[] = {c->k_idx_blocks, c->k_val_blocks, c->v_idx_blocks, c->v_val_blocks};
        for (const void *p : tabs)
            if (!p || ((uintptr_t)p & 7)) return KVQ_ERR_INVALID_ARG;
    }
    if (c->workspace && ((uintptr_t)c->workspace & 15)) return KVQ_ERR_INVALID_ARG;
    if (c->n_sink < 0 || c->n_sink > KVQ_MAX_SINK) return KVQ_ERR_INVALID_ARG;
    if (c->n_sink > 0 && (!c->sink_k || !c->sink_v || ((uintptr_t)c->sink_k & 15) || ((uintptr_t)c->sink_v & 15)))
        return KVQ_ERR_INVALID_ARG;
    return KVQ_OK;
}

static inline KvqSparseFlat kvq_flat_k(const kvq_cache *c) { return KvqSparseFlat{c->k_idx, c->k_val}; }
static inline KvqSparseFlat kvq_flat_v(const kvq_cache *c) { return KvqSparseFlat{c->v_idx, c->v_val}; }
static inline KvqSparseBlocked kvq_blocked_k(const kvq_cache *c)
{
    return KvqSparseBlocked{c->k_idx_blocks, c->k_val_blocks, c->nnz_block_shift};
}
static inline KvqSparseBlocked kvq_blocked_v(const kvq_cache *c)
{
    return KvqSparseBlocked{c->v_idx_blocks, c->v_val_blocks, c->nnz_block_shift};
}
