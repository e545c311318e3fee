// Attention scores against the quantized, pre-RoPE Key cache (paper Sec. 3.2, 3.7, App. "RoPE
// Equation", App. "Kernel Implementation Details"): dense look-up-table mat-vec with the rotary
// embedding applied after de-quantisation, plus the sparse outlier mat-vec, merged in one call.
//
// Design (gfx950).  RoPE rotates channel i with channel i+64, so for one (token n, query head) the
// contribution of that channel pair is   A cos(n theta_i) + B sin(n theta_i)   with
//     A = q_i k_i + q_{i+64} k_{i+64},   B = q_{i+64} k_i - q_i k_{i+64},   k_c = s_c lut[code_c] + z_c.
// A and B depend on the token only through the two codes, which the storage format keeps side by
// side in one 2b-bit field.  Each workgroup therefore builds, per query head and channel pair, a
// table of (A,B) for every code pair in LDS (fp32 pairs, query, scale and zero-point folded in), and
// the hot loop per (token, head, pair) is: extract a field, one 8-byte LDS gather, two fp32 FMAs
// with the cos/sin of the token's angle.  (fp16 table entries would halve the LDS footprint, but
// their 2^-11 relative rounding leaves the scores only just inside a 1e-3 tolerance.)  cos/sin are
// computed once per (token, pair) and shared by all query heads the workgroup handles.  Lanes are
// tokens; a wavefront reads 1 KiB of contiguous codes per load instruction, and the 16-byte pieces
// of the next token tile are requested as soon as the current tile no longer needs the registers
// they land in, so HBM latency hides behind the table look-ups.  For 4-bit codes the joint table
// would have 256 entries, so A and B are split into a part indexed by each code (two 16-entry
// gathers).
//
// The sparse outliers are handled by a second, balanced kernel (lanes = outlier entries) launched
// in front of the dense one in the same call: it writes its per-(head, token) sums to the score
// buffer and the dense kernel adds its own part, so one call yields one merged result.  Attention-
// sink tokens (paper Sec. 3.5), if any, are scored last from their fp16 rows.
#include <stdlib.h>
#include <atomic>
#include <utility>
#include "kvq_common.hpp"
#include "kvq_qk_sparse.hpp"

// Tuning knobs of the piece-major 3-bit kernel (kvq_qk3_kernel): tiles per block, fields per gather group.
#ifndef KVQ_QK3_ENABLE
#define KVQ_QK3_ENABLE 1
#endif
#ifndef KVQ_QK3_TT
#define KVQ_QK3_TT 4
#endif
#ifndef KVQ_QK3_PG
#define KVQ_QK3_PG 4
#endif
#ifndef KVQ_ROTATE_PRIORITY
#define KVQ_ROTATE_PRIORITY 1
#endif


namespace {

template <int BITS>
struct QkCfg {
    static constexpr bool JOINT = BITS <= 3;
    static constexpr int NE = 1 << BITS;
    static constexpr int ENTRIES = JOINT ? (1 << (2 * BITS)) : 2 * NE;   // (A,B) entries per (head, pair)
    static constexpr int CW = 4 * BITS;                                  // dwords per chunk
};

// The chunk of one (token, head) is consumed front to back, so only two of its 16-byte pieces need to
// be in registers at a time: piece j lives in slot j & 1 (4 dwords each).  Dword `wi` of the chunk:
__device__ __forceinline__ uint32_t chunk_dword(const uint32_t (&Wg)[8], int wi)
{
    return Wg[((wi >> 2) & 1) * 4 + (wi & 3)];
}

// Byte offset (field value * 8) of field `i` of a chunk, for indexing a table of 8-byte entries.
template <int FBITS>   // field width in bits
__device__ __forceinline__ uint32_t field_shifted(const uint32_t (&Wg)[8], int i)
{
    // the field, moved to bit 3 (so that, masked, it is a byte offset into 8-byte entries)
    const int bit = i * FBITS, wi = bit >> 5, sh = bit & 31;
    if (sh + FBITS <= 32) {
        if (sh >= 3) return chunk_dword(Wg, wi) >> (sh - 3);
        return chunk_dword(Wg, wi) << (3 - sh);
    }
    return __builtin_amdgcn_alignbit(chunk_dword(Wg, wi + 1), chunk_dword(Wg, wi), sh - 3);
}

// PAIR_GROUP consecutive channel pairs of the dense part for one token.  Written gathers-first so
// that a group's LDS gathers are all in flight before the arithmetic that consumes them:
//   1. per KV head one field extraction per pair, per query head one gather,
//   2. the group's angles -> (cos, sin), shared by all query heads,
//   3. two fp32 FMAs per (pair, query head) and table part.
// G0 is a compile-time constant so that all register-array indices fold.
template <int BITS, int KVH, int RQ, int PAIR_GROUP, int G0>
__device__ __forceinline__ void qk_group(uint32_t (&W)[KVH][8], float (&acc)[KVH * RQ],
                                         const float2_t *tab, float nf, float wave_base, const KvqParamsHeader *hdr,
                                         const uint8_t *cur_chunk, const uint8_t *next_chunk, int64_t plane,
                                         bool valid, bool next_valid)
{
    // nf: this lane's index inside its wavefront (as float); wave_base: lane i holds the reduced angle
    // (in revolutions) of channel pair i at the wavefront's first token
    using C = QkCfg<BITS>;
    constexpr int QH = KVH * RQ, R = RQ;
    constexpr int NE = C::NE;
    constexpr int ENT = C::ENTRIES;
    constexpr int NG = C::JOINT ? 1 : 2;          // gathers per (pair, query head)
    float2_t t[PAIR_GROUP][QH][NG];
#pragma unroll
    for (int p = 0; p < PAIR_GROUP; ++p) {
        const int I = G0 * PAIR_GROUP + p;
#pragma unroll
        for (int g = 0; g < KVH; ++g) {
            uint32_t sh[NG];
            constexpr uint32_t M = ((C::JOINT ? (1u << (2 * BITS)) : (1u << BITS)) - 1u) << 3;
            if (C::JOINT) sh[0] = field_shifted<2 * BITS>(W[g], I);
            else { sh[0] = field_shifted<BITS>(W[g], 2 * I); sh[NG - 1] = field_shifted<BITS>(W[g], 2 * I + 1); }
            uint32_t off_lo[NG];
            bool have_lo = false;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int qh = g * R + r;
                // LDS instructions reach 64 KiB past their address register; tables further up get the
                // excess folded into the masking instruction instead of an extra add
                const uint32_t base = (uint32_t)((qh * 64 + I) * ENT) * 8u;
                const uint32_t hi = base & ~0xFFFFu;
                const uint8_t *tb = (const uint8_t *)tab + (base - hi);
                if (hi == 0) {
                    if (!have_lo) {
#pragma unroll
                        for (int k = 0; k < NG; ++k) off_lo[k] = sh[k] & M;
                        have_lo = true;
                    }
#pragma unroll
                    for (int k = 0; k < NG; ++k) t[p][qh][k] = *(const float2_t *)(tb + k * NE * 8 + off_lo[k]);
                } else {
#pragma unroll
                    for (int k = 0; k < NG; ++k) {
                        const uint32_t off = kvq_and_or(sh[k], M, hi);
                        t[p][qh][k] = *(const float2_t *)(tb + k * NE * 8 + off);
                    }
                }
            }
        }
    }
    float cs[PAIR_GROUP], sn[PAIR_GROUP];
#pragma unroll
    for (int p = 0; p < PAIR_GROUP; ++p) {
        const int I = G0 * PAIR_GROUP + p;
        // angle of pair I at this lane's token = (angle at the wavefront's first token, held by lane I)
        //                                        + lane * theta_I / (2 pi)
        const float base = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wave_base), I));
        const float rev = __builtin_fmaf(nf, hdr->rope_vh[I], base);
        cs[p] = __builtin_amdgcn_cosf(rev);
        sn[p] = __builtin_amdgcn_sinf(rev);
    }
#pragma unroll
    for (int p = 0; p < PAIR_GROUP; ++p)
#pragma unroll
        for (int qh = 0; qh < QH; ++qh)
#pragma unroll
            for (int k = 0; k < NG; ++k) {
                acc[qh] = __builtin_fmaf(t[p][qh][k].x, cs[p], acc[qh]);
                acc[qh] = __builtin_fmaf(t[p][qh][k].y, sn[p], acc[qh]);
            }
    // Pin the accumulators: an empty asm that "modifies" them and clobbers memory keeps the compiler
    // from hoisting later groups' gathers above this point (register pressure) or sinking this
    // group's arithmetic below later gathers.
#pragma unroll
    for (int qh = 0; qh < QH; ++qh) asm volatile("" : "+v"(acc[qh]) : : "memory");
    // Software pipelining: a 16-byte piece of the chunk is dead once the last field that touches it
    // has been consumed; the piece two positions further down the stream (of this tile, or of the
    // next tile once this one runs out) is requested into its register slot right away, so every
    // load has a third of a tile's arithmetic to hide behind.
    constexpr int FB = 2 * BITS;
    constexpr int first_field = G0 * PAIR_GROUP, last_field = first_field + PAIR_GROUP - 1;
#pragma unroll
    for (int j = 0; j < BITS; ++j) {
        const int last_user = (128 * (j + 1) - 1) / FB;      // last field with a bit in piece j
        if (last_user >= first_field && last_user <= last_field) {
            const int jn = j + 2;                            // stream position of the piece to fetch
            if (jn < BITS) {
                if (valid) {
#pragma unroll
                    for (int g = 0; g < KVH; ++g) {
                        const uint4 v = kvq_load_stream16(cur_chunk + g * plane + jn * 1024);
                        W[g][(jn & 1) * 4 + 0] = v.x; W[g][(jn & 1) * 4 + 1] = v.y;
                        W[g][(jn & 1) * 4 + 2] = v.z; W[g][(jn & 1) * 4 + 3] = v.w;
                    }
                }
            } else if (jn - BITS == 0 || (BITS & 1) == 0) {
                // next tile's piece 0 (or, for an even piece count, also its piece 1) lands in the slot just freed
                const int jt = jn - BITS;
                if (next_valid) {
#pragma unroll
                    for (int g = 0; g < KVH; ++g) {
                        const uint4 v = kvq_load_stream16(next_chunk + g * plane + jt * 1024);
                        W[g][(j & 1) * 4 + 0] = v.x; W[g][(j & 1) * 4 + 1] = v.y;
                        W[g][(j & 1) * 4 + 2] = v.z; W[g][(j & 1) * 4 + 3] = v.w;
                    }
                }
            }
            // odd piece count, last piece: handled at the end of the tile (the slots swap roles there)
        }
    }
}

template <int BITS, int KVH, int RQ, int PG, int... G>
__device__ __forceinline__ void qk_all_pairs(std::integer_sequence<int, G...>,
                                             uint32_t (&W)[KVH][8], float (&acc)[KVH * RQ],
                                             const float2_t *tab, float nf, float wave_base,
                                             const KvqParamsHeader *hdr, const uint8_t *cur_chunk,
                                             const uint8_t *next_chunk, int64_t plane, bool valid, bool next_valid)
{
    (qk_group<BITS, KVH, RQ, PG, G>(W, acc, tab, nf, wave_base, hdr, cur_chunk, next_chunk, plane, valid, next_valid), ...);
}

// Stage the scaled query and the per-channel (scale, zero-point) of the workgroup's heads in LDS and
// build the (A,B) tables from them.  A table (one query head, one channel pair) has ENT entries; ENT
// lanes of a wavefront fill it, one entry each, so a lane's signposts are loop constants and LDS
// writes are conflict-free.  Ends with a workgroup barrier.
template <int BITS, int KVH, int RQ, int NT>
__device__ __forceinline__ void qk_build_tables(float2_t *tab, float *qs, float2_t *szs, const KvqParamsView &pv,
                                                const float *__restrict__ q_rot, float scale, int q0, int kv0)
{
    using C = QkCfg<BITS>;
    constexpr int QH = KVH * RQ, R = RQ;
    constexpr int NE = C::NE;
    constexpr int ENT = C::ENTRIES;
    const int tid = threadIdx.x;
    for (int j = tid; j < QH * 128; j += NT) qs[j] = q_rot[(int64_t)q0 * 128 + j] * scale;
    for (int j = tid; j < KVH * 128; j += NT) szs[j] = float2_t{pv.s[kv0 * 128 + j], pv.z[kv0 * 128 + j]};
    __syncthreads();
    constexpr int TW = 64 / ENT;                     // tables per wavefront step
    constexpr int NWAVES = NT / 64;
    constexpr int STEP = NWAVES * TW;                // tables per workgroup step
    static_assert(64 % STEP == 0 || STEP % 64 == 0, "table build assumes the step divides the pair count");
    const int lane = tid & 63, wave = tid >> 6;
    const int f = lane % ENT, sub = lane / ENT;
    float lut_a = 0.f, lut_b = 0.f;                  // joint: signposts of the two codes; split: lut_a only
#pragma unroll
    for (int j = 0; j < NE; ++j) {
        const float v = pv.hdr->lut_k[j];
        if ((f & (NE - 1)) == j) lut_a = v;
        if (C::JOINT && (f >> BITS) == j) lut_b = v;
    }
    const bool upper = !C::JOINT && f >= NE;         // split tables: second half belongs to channel i+64
    for (int tb = wave * TW + sub; tb < QH * 64; tb += STEP) {
        const int qh = tb >> 6, i = tb & 63;
        const float2_t lo = szs[(qh / R) * 128 + i], hi = szs[(qh / R) * 128 + i + 64];
        const float qa = qs[qh * 128 + i], qb = qs[qh * 128 + i + 64];
        float a, b;
        if (C::JOINT) {
            const float klo = __builtin_fmaf(lo.x, lut_a, lo.y), khi = __builtin_fmaf(hi.x, lut_b, hi.y);
            a = qa * klo + qb * khi;
            b = qb * klo - qa * khi;
        } else {
            const float k = upper ? __builtin_fmaf(hi.x, lut_a, hi.y) : __builtin_fmaf(lo.x, lut_a, lo.y);
            a = upper ? qb * k : qa * k;
            b = upper ? -qa * k : qb * k;
        }
        tab[tb * ENT + f] = float2_t{a, b};
    }
    __syncthreads();
}

// KVH KV heads per workgroup, RQ query heads per KV head handled here (RQ divides the model's GQA
// ratio `r`; when RQ < r several workgroups share a KV head), PG channel pairs per gather group.
template <int BITS, int KVH, int RQ, int NT, int PG, bool STATS, bool SPAN = false>
__global__ __launch_bounds__(NT) void kvq_qk_kernel(const void *__restrict__ params, int D, int r,
                                                    int64_t cap, int64_t L, const uint8_t *__restrict__ k_codes,
                                                    const float *__restrict__ q_rot, float scale,
                                                    float *__restrict__ scores, int64_t ld, int n_tiles,
                                                    int add_prev, float *__restrict__ stat_slots, int n_sink,
                                                    unsigned long long *span)
{
    // SPAN: timing-aid instantiation (kvq_profile_*): the workgroup leaves its start and end times in
    // `span`.  A separate instantiation, and none for the eight-head variants: they have no register
    // to spare for the pointer, and the variant that is timed should be the one that is used.
    if (SPAN) kvq_span_start(span);
    // add_prev != 0: the score buffer already holds the sparse part; add to it instead of overwriting.
    // STATS: the workgroup also leaves the maximum of the scores it wrote (tokens below n_sink
    // excepted: the attention-sink kernel replaces their scores) in slot blockIdx.x of each of its
    // query heads.  A separate instantiation: the running maxima cost a register per head.
    using C = QkCfg<BITS>;
    constexpr int QH = KVH * RQ, R = RQ;
    constexpr int NE = C::NE;
    constexpr int ENT = C::ENTRIES;
    // Statically sized LDS (up to 136 KiB of the 160 KiB a gfx950 workgroup may use): with a known base
    // address the table offsets fold into the gathers' immediate offsets.
    __shared__ __attribute__((aligned(16))) float2_t tab[QH * 64 * ENT];  // [QH][64][ENT]
    __shared__ float qs[QH * 128];                                        // query * scale
    __shared__ float2_t szs[(QH / R) * 128];                              // per-channel (scale, zero-point)

    const KvqParamsView pv = kvq_params_view(params, D);
    const int tid = threadIdx.x;
    const int q0 = blockIdx.y * QH;
    const int kv0 = q0 / r;

    qk_build_tables<BITS, KVH, RQ, NT>(tab, qs, szs, pv, q_rot, scale, q0, kv0);

    // ---- token tiles (software-pipelined over the workgroup's tiles) -------------------------
    const int64_t plane = cap * 16 * BITS;                 // bytes between consecutive KV heads
    // the workgroups of a head group split the tiles as evenly as possible
    const int tile_begin = (int)(((int64_t)blockIdx.x * n_tiles) / gridDim.x);
    const int tile_end = (int)(((int64_t)(blockIdx.x + 1) * n_tiles) / gridDim.x);
    const int tiles_per_wg = tile_end - tile_begin;
    int64_t n = (int64_t)tile_begin * NT + tid;
    bool valid = n < L;
    const float my_vh = pv.hdr->rope_vh[tid & 63], my_vl = pv.hdr->rope_vl[tid & 63];   // this lane's pair
    uint32_t W[KVH][8];                                    // two 16-byte pieces per KV head
    const uint8_t *cur_chunk = k_codes + kvq_k_piece0(BITS, cap, valid ? n : 0, kv0);
    if (valid) {
#pragma unroll
        for (int g = 0; g < KVH; ++g)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const uint4 v = kvq_load_stream16(cur_chunk + g * plane + j * 1024);
                W[g][4 * j + 0] = v.x; W[g][4 * j + 1] = v.y; W[g][4 * j + 2] = v.z; W[g][4 * j + 3] = v.w;
            }
    }
    // STATS: running maxima of the scores written.  With eight query heads per thread there is no
    // register for them: the wavefront's maxima then live in LDS slots of its own (the staged query's
    // array, dead once the tables are built; only lane 0 of the wavefront touches its slots) and are
    // brought up to date after every tile.
    constexpr bool STAT_LDS = STATS && QH >= 8;
    float stat_m[(STATS && !STAT_LDS) ? QH : 1];
    if (STATS && !STAT_LDS) {
#pragma unroll
        for (int qh = 0; qh < QH; ++qh) stat_m[qh] = KVQ_STAT_FLOOR;
    }
    if (STAT_LDS && (tid & 63) == 0) {
#pragma unroll
        for (int qh = 0; qh < QH; ++qh) qs[(tid >> 6) * QH + qh] = KVQ_STAT_FLOOR;
    }
    for (int tile = 0; tile < tiles_per_wg; ++tile) {
        // wavefronts w, w + 4, ... of the workgroup share a SIMD: each takes every priority in turn
        if (KVQ_ROTATE_PRIORITY) kvq_set_wave_priority(__builtin_amdgcn_readfirstlane(tid >> 8) + tile);
        const int64_t nn = n + NT;
        const bool next_valid = (tile + 1 < tiles_per_wg) && (nn < L);
        const uint8_t *next_chunk = k_codes + kvq_k_piece0(BITS, cap, next_valid ? nn : n, kv0);
        // lane i reduces the angle of channel pair i at the wavefront's first token (n - lane, a multiple
        // of 64); every lane then needs one FMA per pair instead of its own reduction
        const int lane_id = tid & 63;
        const float nf = (float)lane_id;
        const float wave_base = rope_rev((float)(n - lane_id), my_vh, my_vl);
        // the sparse part of the scores: requested before the tile's arithmetic and consumed after it
        // when the registers allow; with eight query heads per thread they do not, and the loads wait
        // until the arithmetic is done (other wavefronts cover the latency)
        constexpr bool PREV_EARLY = QH < 8;
        float acc[QH], prev[QH];
#pragma unroll
        for (int qh = 0; qh < QH; ++qh) {
            acc[qh] = 0.f;
            if (PREV_EARLY) prev[qh] = (add_prev && valid) ? scores[(int64_t)(q0 + qh) * ld + n] : 0.f;
        }
        // lanes past the end run the arithmetic on whatever their registers hold (table offsets are
        // masked, so every gather stays inside the table) and simply skip loads and stores
        // a wavefront whose 64 tokens all lie past the end (ragged last tile) skips the arithmetic
        if (__ballot(valid) != 0ull)
            qk_all_pairs<BITS, KVH, RQ, PG>(std::make_integer_sequence<int, 64 / PG>{}, W, acc, tab, nf, wave_base,
                                            pv.hdr, cur_chunk, next_chunk, plane, valid, next_valid);
        if (BITS & 1) {
            // odd piece count: the next tile's piece 0 arrived in slot 1; move it to slot 0 (whose last
            // occupant is dead now) and request the next tile's piece 1 into slot 1
#pragma unroll
            for (int g = 0; g < KVH; ++g) {
#pragma unroll
                for (int k = 0; k < 4; ++k) W[g][k] = W[g][4 + k];
                if (next_valid) {
                    const uint4 v = kvq_load_stream16(next_chunk + g * plane + 1024);
                    W[g][4] = v.x; W[g][5] = v.y; W[g][6] = v.z; W[g][7] = v.w;
                }
            }
        }
        if (!PREV_EARLY) {
#pragma unroll
            for (int qh = 0; qh < QH; ++qh) {
                asm volatile("" : "+v"(acc[qh]));      // keeps the loads below the arithmetic
                prev[qh] = (add_prev && valid) ? scores[(int64_t)(q0 + qh) * ld + n] : 0.f;
            }
        }
        if (valid) {
#pragma unroll
            for (int qh = 0; qh < QH; ++qh) {
                const float x = acc[qh] + prev[qh];
                scores[(int64_t)(q0 + qh) * ld + n] = x;
                if (STATS && !STAT_LDS && n >= n_sink)
                    stat_m[(STATS && !STAT_LDS) ? qh : 0] = __builtin_fmaxf(stat_m[(STATS && !STAT_LDS) ? qh : 0], x);
                acc[qh] = x;
            }
        }
        if (STAT_LDS) {
            float *wst = qs + (tid >> 6) * QH;
#pragma unroll
            for (int qh = 0; qh < QH; ++qh) {
                const float w = kvq_wave_max((valid && n >= n_sink) ? acc[qh] : KVQ_STAT_FLOOR);
                if ((tid & 63) == 0) wst[qh] = __builtin_fmaxf(wst[qh], w);
            }
        }
        n = nn;
        valid = next_valid;
        cur_chunk = next_chunk;
    }
    if (STATS) {
        // workgroup-wide maximum per query head: wavefronts first, then one thread per head over the
        // wavefronts' values (the staged query is dead by now: its array holds them)
        float *wst = qs;                                      // [NT / 64][QH]
        if (!STAT_LDS) {
#pragma unroll
            for (int qh = 0; qh < QH; ++qh) {
                const float w = kvq_wave_max(stat_m[(STATS && !STAT_LDS) ? qh : 0]);
                if ((tid & 63) == 0) wst[(tid >> 6) * QH + qh] = w;
            }
        }
        __syncthreads();
        if (tid < QH) {
            float m = KVQ_STAT_FLOOR;
#pragma unroll
            for (int w = 0; w < NT / 64; ++w) m = __builtin_fmaxf(m, wst[w * QH + tid]);
            stat_slots[(int64_t)(q0 + tid) * KVQ_STAT_SLOTS + blockIdx.x] = m;
        }
    }
    if (SPAN) kvq_span_end(span);
}

// ---- piece-major dense kernel for 3-bit codes ------------------------------------------------------
// The kernel above computes cos / sin of every (token, channel pair) with the hardware's quarter-rate
// instructions: 11 of the ~30 issue slots a lane spends on a pair for four query heads.  Here a lane
// owns TT tokens, one in each of TT consecutive tiles (KVQ_ROPE_STEP positions apart), and only the
// first one's (cos, sin) come from v_cos / v_sin: each further one is the previous one rotated by the
// wavefront-uniform angle KVQ_ROPE_STEP * theta_i (two multiplies and two multiply-adds with constants
// from scalar registers).  To keep the pairs' (cos, sin) in registers from tile to tile the loops are
// piece-major: for each 16-byte piece of the chunk (21 or 22 fields), for each of the TT tiles, the
// piece of that tile's token is consumed; the partial sums of the TT x QH scores stay in registers
// until all pieces are done.  HBM is still read once, in the same 1 KiB segments.
// A 6-bit field is consumed in the pass of the piece that holds its last bit; fields 21 and 42 start in
// the piece before (2 and 4 bits), which are carried over packed in three registers.
constexpr int PM_FB = 6;                                                  // field width, bits
__host__ __device__ constexpr int pm_pass_of(int i) { return (PM_FB * i + PM_FB - 1) / 128; }
__host__ __device__ constexpr int pm_first(int j)                         // first field of pass j (64 for j = 3)
{
    int i = 0;
    while (i < 64 && pm_pass_of(i) < j) ++i;
    return i;
}
constexpr int PM_MAXF = 22;                                               // most fields in a pass
static_assert(pm_first(1) == 21 && pm_first(2) == 42 && pm_first(3) == 64, "3-bit chunk: 21 + 21 + 22 fields");

// Field at bit position `bit` (>= 0) of the piece P, moved to bit 3 (unmasked).
__device__ __forceinline__ uint32_t pm_field_shifted(const uint32_t (&P)[4], int bit)
{
    const int wi = bit >> 5, sh = bit & 31;
    if (sh + PM_FB <= 32) {
        if (sh >= 3) return P[wi] >> (sh - 3);
        return P[wi] << (3 - sh);
    }
    return __builtin_amdgcn_alignbit(P[wi + 1], P[wi], sh - 3);
}

// PG consecutive fields (first one: number G0 * PG of pass J) of tile T for all heads of the workgroup.
template <int KVH, int RQ, int TT, int PG, int J, int T, int G0>
__device__ __forceinline__ void pm_group(const uint32_t (&P)[KVH][4], float (&acc)[TT * KVH * RQ],
                                         float (&cs)[PM_MAXF], float (&sn)[PM_MAXF], const uint32_t (&carry)[3],
                                         const float2_t *tab, float nf, float wave_base,
                                         const KvqParamsHeader *hdr)
{
    constexpr int QH = KVH * RQ, R = RQ, ENT = 64;
    constexpr int F0 = pm_first(J), NF = pm_first(J + 1) - F0;
    constexpr uint32_t M = 63u << 3;
    float2_t t[PG][QH];
#pragma unroll
    for (int p = 0; p < PG; ++p) {
        const int k = G0 * PG + p;
        if (k < NF) {
            const int I = F0 + k, bit = PM_FB * I - 128 * J;              // bit < 0: the field starts in the piece before
#pragma unroll
            for (int g = 0; g < KVH; ++g) {
                uint32_t sh;
                if (bit >= 0) {
                    sh = pm_field_shifted(P[g], bit);
                } else {
                    // low -bit bits come from the carry of (tile T, head g), the rest from this piece
                    const int nb = -bit, idx = T * KVH + g;
                    uint32_t c;
                    if (J == 1) c = __builtin_amdgcn_ubfe(carry[0], 2 * idx, 2);
                    else c = __builtin_amdgcn_ubfe(carry[1 + (idx >> 3)], 4 * (idx & 7), 4);
                    sh = ((P[g][0] << nb) | c) << 3;
                }
                uint32_t off_lo = 0;
                bool have_lo = false;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int qh = g * R + r;
                    const uint32_t base = (uint32_t)((qh * 64 + I) * ENT) * 8u;
                    const uint32_t hi = base & ~0xFFFFu;
                    const uint8_t *tb = (const uint8_t *)tab + (base - hi);
                    if (hi == 0) {
                        if (!have_lo) { off_lo = sh & M; have_lo = true; }
                        t[p][qh] = *(const float2_t *)(tb + off_lo);
                    } else {
                        t[p][qh] = *(const float2_t *)(tb + kvq_and_or(sh, M, hi));
                    }
                }
            }
        }
    }
#pragma unroll
    for (int p = 0; p < PG; ++p) {
        const int k = G0 * PG + p;
        if (k < NF) {
            const int I = F0 + k;
            if (T == 0) {
                const float base = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wave_base), I));
                const float rev = __builtin_fmaf(nf, hdr->rope_vh[I], base);
                cs[k] = __builtin_amdgcn_cosf(rev);
                sn[k] = __builtin_amdgcn_sinf(rev);
            } else {
                // (cos, sin) advance by KVQ_ROPE_STEP positions, in place: written as instructions so that
                // the results stay in the registers of the operands (otherwise every tile ends with a
                // block of register copies)
                const float cd = hdr->rope_cd[I], sd = hdr->rope_sd[I];
                const float t1 = sn[k] * sd, t2 = cs[k] * sd;
                asm("v_fma_f32 %0, %0, %1, -%2" : "+v"(cs[k]) : "s"(cd), "v"(t1));
                asm("v_fma_f32 %0, %0, %1, %2" : "+v"(sn[k]) : "s"(cd), "v"(t2));
            }
        }
    }
#pragma unroll
    for (int p = 0; p < PG; ++p) {
        const int k = G0 * PG + p;
        if (k < NF) {
#pragma unroll
            for (int qh = 0; qh < QH; ++qh) {
                acc[T * QH + qh] = __builtin_fmaf(t[p][qh].x, cs[k], acc[T * QH + qh]);
                acc[T * QH + qh] = __builtin_fmaf(t[p][qh].y, sn[k], acc[T * QH + qh]);
            }
        }
    }
    // keeps the groups in order (see qk_group)
#pragma unroll
    for (int qh = 0; qh < QH; ++qh) asm volatile("" : "+v"(acc[T * QH + qh]) : : "memory");
}

template <int KVH, int RQ, int TT, int PG, int J, int T, int... G>
__device__ __forceinline__ void pm_groups(std::integer_sequence<int, G...>, const uint32_t (&P)[KVH][4],
                                          float (&acc)[TT * KVH * RQ], float (&cs)[PM_MAXF], float (&sn)[PM_MAXF],
                                          const uint32_t (&carry)[3], const float2_t *tab, float nf, float wave_base,
                                          const KvqParamsHeader *hdr)
{
    (pm_group<KVH, RQ, TT, PG, J, T, G>(P, acc, cs, sn, carry, tab, nf, wave_base, hdr), ...);
}

// Stage S = J * TT + T of a block: piece J of tile T.  The piece sits in W[S & 1]; the next stage's
// piece (this block's, or piece 0 of the next block's first tile) is requested into the other slot
// before the arithmetic starts.  Addresses are a wavefront-uniform base plus 32-bit offsets (the
// launcher checks that the codes are smaller than 4 GiB).
template <int KVH, int RQ, int TT, int PG, int S>
__device__ __forceinline__ void pm_stage(uint32_t (&W)[2][KVH][4], float (&acc)[TT * KVH * RQ], float (&cs)[PM_MAXF],
                                         float (&sn)[PM_MAXF], uint32_t (&carry)[3], const float2_t *tab, float nf,
                                         float wave_base, const KvqParamsHeader *hdr,
                                         const uint8_t *__restrict__ k_codes, uint32_t off0, uint32_t plane,
                                         uint32_t vm, uint32_t any, bool next_block_valid)
{
    // off0: byte offset of piece 0 of this lane's token in tile 0 of the block, KV head 0 of the
    // workgroup; tile t is KVQ_ROPE_STEP tokens = 16 blocks of 64 tokens further on.  vm: this lane's
    // valid tiles (bit t); any: tiles with a valid token in this wavefront (uniform).
    constexpr int J = S / TT, T = S % TT, LAST = 3 * TT - 1;
    constexpr uint32_t TILE_BYTES = (uint32_t)(KVQ_ROPE_STEP / 64) * 64 * 16 * 3;
    // wavefronts w, w + 4, w + 8, w + 12 of the workgroup share a SIMD: each takes every priority in turn
    if (KVQ_ROTATE_PRIORITY) kvq_set_wave_priority(__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 8)) + S);
    if (S < LAST) {
        constexpr int JN = (S + 1) / TT, TN = (S + 1) % TT;
        if ((vm >> TN) & 1u) {
#pragma unroll
            for (int g = 0; g < KVH; ++g) {
                const uint4 v = kvq_load_stream16(k_codes + (off0 + g * plane + (TN * TILE_BYTES + JN * 1024)));
                W[(S + 1) & 1][g][0] = v.x; W[(S + 1) & 1][g][1] = v.y; W[(S + 1) & 1][g][2] = v.z; W[(S + 1) & 1][g][3] = v.w;
            }
        }
    } else if (next_block_valid) {
#pragma unroll
        for (int g = 0; g < KVH; ++g) {
            const uint4 v = kvq_load_stream16(k_codes + (off0 + g * plane + TT * TILE_BYTES));
            W[(S + 1) & 1][g][0] = v.x; W[(S + 1) & 1][g][1] = v.y; W[(S + 1) & 1][g][2] = v.z; W[(S + 1) & 1][g][3] = v.w;
        }
    }
    if ((any >> T) & 1u) {
        if (J < 2) {
            // the top bits of this piece open the first field of the next pass
#pragma unroll
            for (int g = 0; g < KVH; ++g) {
                const int idx = T * KVH + g;
                if (J == 0) carry[0] |= (W[S & 1][g][3] >> 30) << (2 * idx);
                else carry[1 + (idx >> 3)] |= (W[S & 1][g][3] >> 28) << (4 * (idx & 7));
            }
        }
        constexpr int NF = pm_first(J + 1) - pm_first(J);
        pm_groups<KVH, RQ, TT, PG, J, T>(std::make_integer_sequence<int, (NF + PG - 1) / PG>{}, W[S & 1], acc, cs, sn,
                                         carry, tab, nf, wave_base, hdr);
    }
}

// Pass J of a block: piece J of each of the block's TT tiles.  The (cos, sin) of the pass's fields live
// here, from the first tile (computed) to the last (rotated).
template <int KVH, int RQ, int TT, int PG, int J, int... T>
__device__ __forceinline__ void pm_pass(std::integer_sequence<int, T...>, uint32_t (&W)[2][KVH][4],
                                        float (&acc)[TT * KVH * RQ], uint32_t (&carry)[3], const float2_t *tab,
                                        float nf, float wave_base, const KvqParamsHeader *hdr,
                                        const uint8_t *__restrict__ k_codes, uint32_t off0, uint32_t plane,
                                        uint32_t vm, uint32_t any, bool next_block_valid)
{
    float cs[PM_MAXF], sn[PM_MAXF];
    (pm_stage<KVH, RQ, TT, PG, J * TT + T>(W, acc, cs, sn, carry, tab, nf, wave_base, hdr, k_codes, off0, plane, vm,
                                           any, next_block_valid), ...);
}

// Timing aid of the piece-major kernel.  The kernel has no register to carry a pointer, or a slot
// number, through its loops (an instantiation that took the slots as an argument spilled around them
// and ran 15 % slower than the kernel it was meant to time), so the address of the launch's span
// slots lives in device memory and is loaded where it is used, once before the first and once after
// the last instruction of the kernel proper, and the workgroups share one pair of words: the earliest
// start (an atomic minimum) and the latest end (an atomic maximum).  Null (the normal state): nothing
// is stamped.  The host stores the address, and resets the launch's slots, with a small kernel on the
// launch stream before every launch whose span is taken, and once more when spans are switched off.
__device__ unsigned long long *kvq_qk3_span_slots = nullptr;
__global__ void kvq_qk3_set_span(unsigned long long *slots)
{
    if (threadIdx.x == 0) kvq_qk3_span_slots = slots;
    if (slots) {                                   // pair 0: (earliest start, latest end); the rest unused
        slots[2 * threadIdx.x] = threadIdx.x == 0 ? ~0ull : 0ull;
        slots[2 * threadIdx.x + 1] = 0ull;
    }
}
__device__ __forceinline__ unsigned long long *qk3_span_slots_now()
{
    unsigned long long *p = *(unsigned long long *volatile *)&kvq_qk3_span_slots;
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return (unsigned long long *)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ void qk3_span_start()
{
    unsigned long long *sp = qk3_span_slots_now();
    if (sp && threadIdx.x == 0)
        __hip_atomic_fetch_min(sp, (unsigned long long)wall_clock64(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Every thread of the workgroup must call this (it holds a barrier when spans are being taken).
__device__ __forceinline__ void qk3_span_end()
{
    unsigned long long *sp = qk3_span_slots_now();
    if (sp) {
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");     // this wavefront's stores are acknowledged
        __syncthreads();
        if (threadIdx.x == 0)
            __hip_atomic_fetch_max(sp + 1, (unsigned long long)wall_clock64(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Same arguments, grid and results as kvq_qk_kernel<3, KVH, RQ, 1024, ...>; tiles are KVQ_ROPE_STEP tokens.
template <int KVH, int RQ, int TT, int PG, bool STATS, bool SPAN = false>
__global__ __launch_bounds__(KVQ_ROPE_STEP) void kvq_qk3_kernel(const void *__restrict__ params, int D, int r,
                                                               int64_t cap, int64_t L,
                                                               const uint8_t *__restrict__ k_codes,
                                                               const float *__restrict__ q_rot, float scale,
                                                               float *__restrict__ scores, int64_t ld, int n_tiles,
                                                               int add_prev, float *__restrict__ stat_slots,
                                                               int n_sink, unsigned long long *)
{
    qk3_span_start();
    constexpr int BITS = 3, NT = KVQ_ROPE_STEP;
    static_assert(KVH * TT <= 16, "the carried bits of a block are packed in 32 + 64 bits");
    constexpr int QH = KVH * RQ, R = RQ, ENT = 64;
    __shared__ __attribute__((aligned(16))) float2_t tab[QH * 64 * ENT];  // [QH][64][ENT]
    __shared__ float qs[QH * 128];                                        // query * scale
    __shared__ float2_t szs[(QH / R) * 128];                              // per-channel (scale, zero-point)

    const KvqParamsView pv = kvq_params_view(params, D);
    const int tid = threadIdx.x;
    const int q0 = blockIdx.y * QH;
    const int kv0 = q0 / r;
    const uint32_t plane = (uint32_t)(cap * 16 * BITS);    // bytes between consecutive KV heads
    const int tile_begin = (int)(((int64_t)blockIdx.x * n_tiles) / gridDim.x);
    const int tile_end = (int)(((int64_t)(blockIdx.x + 1) * n_tiles) / gridDim.x);
    const int lane_id = tid & 63;
    const float nf = (float)lane_id;
    // the first piece of the first tile is requested before anything else
    uint32_t W[2][KVH][4];
    int64_t n0 = (int64_t)tile_begin * NT + tid;           // this lane's token in the block's first tile
    if (tile_begin < tile_end && n0 < L) {
        const uint32_t off = (uint32_t)kvq_k_piece0(BITS, cap, n0, kv0);
#pragma unroll
        for (int g = 0; g < KVH; ++g) {
            const uint4 v = kvq_load_stream16(k_codes + (off + g * plane));
            W[0][g][0] = v.x; W[0][g][1] = v.y; W[0][g][2] = v.z; W[0][g][3] = v.w;
        }
    }
    qk_build_tables<BITS, KVH, RQ, NT>(tab, qs, szs, pv, q_rot, scale, q0, kv0);
    const float my_vh = pv.hdr->rope_vh[lane_id], my_vl = pv.hdr->rope_vl[lane_id];   // this lane's pair
    // STATS: a wavefront keeps the maxima of the scores it wrote in LDS slots of its own (the staged
    // query's array, dead by now; only lane 0 of the wavefront touches its slots: no atomics)
    float *wst = qs + (tid >> 6) * QH;                     // [NT / 64][QH]
    if (STATS && lane_id == 0) {
#pragma unroll
        for (int qh = 0; qh < QH; ++qh) wst[qh] = KVQ_STAT_FLOOR;
    }
    for (int tile0 = tile_begin; tile0 < tile_end; tile0 += TT) {
        const int nt_blk = (tile_end - tile0 < TT) ? tile_end - tile0 : TT;
        uint32_t vm = 0, any = 0;
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            const bool v = t < nt_blk && n0 + (int64_t)t * NT < L;
            vm |= v ? (1u << t) : 0u;
            any |= (__ballot(v) != 0ull) ? (1u << t) : 0u;
        }
        const bool next_block_valid = tile0 + TT < tile_end && n0 + (int64_t)TT * NT < L;
        // (a lane past the end of the context keeps an offset inside the array; it is never loaded from)
        const uint32_t off0 = (uint32_t)kvq_k_piece0(BITS, cap, (vm & 1u) ? n0 : 0, kv0);
        // lane i reduces the angle of channel pair i at the wavefront's first token of the block's first tile
        const float wave_base = rope_rev((float)(n0 - lane_id), my_vh, my_vl);
        float acc[TT * QH];
        uint32_t carry[3] = {0u, 0u, 0u};
#pragma unroll
        for (int a = 0; a < TT * QH; ++a) acc[a] = 0.f;
        pm_pass<KVH, RQ, TT, PG, 0>(std::make_integer_sequence<int, TT>{}, W, acc, carry, tab, nf, wave_base, pv.hdr,
                                    k_codes, off0, plane, vm, any, next_block_valid);
        pm_pass<KVH, RQ, TT, PG, 1>(std::make_integer_sequence<int, TT>{}, W, acc, carry, tab, nf, wave_base, pv.hdr,
                                    k_codes, off0, plane, vm, any, next_block_valid);
        pm_pass<KVH, RQ, TT, PG, 2>(std::make_integer_sequence<int, TT>{}, W, acc, carry, tab, nf, wave_base, pv.hdr,
                                    k_codes, off0, plane, vm, any, next_block_valid);
        // the next block's first piece arrived in slot (3 * TT) & 1; the block expects it in slot 0
        if ((3 * TT) & 1) {
#pragma unroll
            for (int g = 0; g < KVH; ++g)
#pragma unroll
                for (int k = 0; k < 4; ++k) W[0][g][k] = W[1][g][k];
        }
        // scores of the block: the sparse part (if any) is loaded now and added
        float prev[TT * QH];
#pragma unroll
        for (int t = 0; t < TT; ++t)
#pragma unroll
            for (int qh = 0; qh < QH; ++qh)
                prev[t * QH + qh] = (add_prev && ((vm >> t) & 1u)) ? scores[(int64_t)(q0 + qh) * ld + n0 + (int64_t)t * NT] : 0.f;
        float bm[STATS ? QH : 1];                             // maxima of this block's scores
        if (STATS) {
#pragma unroll
            for (int qh = 0; qh < QH; ++qh) bm[qh] = KVQ_STAT_FLOOR;
        }
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            if ((vm >> t) & 1u) {
                const int64_t n = n0 + (int64_t)t * NT;
#pragma unroll
                for (int qh = 0; qh < QH; ++qh) {
                    const float x = acc[t * QH + qh] + prev[t * QH + qh];
                    scores[(int64_t)(q0 + qh) * ld + n] = x;
                    if (STATS && n >= n_sink) bm[STATS ? qh : 0] = __builtin_fmaxf(bm[STATS ? qh : 0], x);
                }
            }
        }
        if (STATS) {
#pragma unroll
            for (int qh = 0; qh < QH; ++qh) {
                const float w = kvq_wave_max(bm[STATS ? qh : 0]);
                if (lane_id == 0) wst[qh] = __builtin_fmaxf(wst[qh], w);
            }
        }
        n0 += (int64_t)TT * NT;
    }
    if (STATS) {
        __syncthreads();
        if (tid < QH) {
            float m = KVQ_STAT_FLOOR;
#pragma unroll
            for (int w = 0; w < NT / 64; ++w) m = __builtin_fmaxf(m, qs[w * QH + tid]);
            stat_slots[(int64_t)(q0 + tid) * KVQ_STAT_SLOTS + blockIdx.x] = m;
        }
    }
    qk3_span_end();
}

template <int R, int QS_TW, class SP>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8)))
void kvq_qk_sparse(const void *__restrict__ params, int D, int n_q_heads, int64_t L,
                   const uint32_t *__restrict__ k_ptr, const SP ksp, uint32_t nnz_cap,
                   const float *__restrict__ q_rot,
                   float scale, float *__restrict__ scores, int64_t ld, int64_t tokens_per_wave)
{
    qk_sparse_body<R, QS_TW, SP>((int)blockIdx.x, params, D, n_q_heads, L, k_ptr, ksp, nnz_cap, q_rot, scale, scores,
                                 ld, tokens_per_wave);
}

template <int R, int TW, class SP>
kvq_status launch_qk_sparse_tw(const kvq_cache *c, const SP ksp, const float *q, float scale, float *scores, int64_t ld, hipStream_t s)
{
    const int Hq = c->n_q_heads;
    const int64_t L = c->n_tokens_k;
    QkSparsePlan plan;
    if (!qk_sparse_plan(Hq, L, TW, 0, plan)) return KVQ_ERR_UNSUPPORTED;
    // the kernel's dynamic-LDS limit is raised once per instantiation, to the most any launch asks for
    // (initialisation of a function-local static is thread-safe)
    static const hipError_t lds_attr = hipFuncSetAttribute((const void *)kvq_qk_sparse<R, TW, SP>,
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 147456);
    KVQ_HIP_CHECK(lds_attr);
    kvq_qk_sparse<R, TW, SP><<<plan.grid, 64 * plan.waves, plan.lds, s>>>(
        c->params, c->n_kv_heads * KVQ_HEAD_DIM, Hq, L, c->k_ptr, ksp, (uint32_t)c->cap_nnz_k, q, scale, scores, ld,
        plan.tokens_per_wave);
    KVQ_HIP_CHECK(hipGetLastError());
    return KVQ_OK;
}

template <int R>
kvq_status launch_qk_sparse(const kvq_cache *c, const float *q, float scale, float *scores, int64_t ld, hipStream_t s)
{
    if (c->cap_nnz_k >= ((int64_t)1 << 31)) return KVQ_ERR_UNSUPPORTED;      // byte offsets are 32-bit
    // Sub-ranges of 8 tokens keep a wavefront's tile small (many wavefronts per CU), which is what
    // counts when every token brings tens of outliers.  With few outliers per token the cost is the
    // tile itself (cleared, written out as scores, one piece per head and sub-range), and sub-ranges
    // of 32 tokens (128-byte pieces: whole cache lines) are the better trade.  The array capacity per
    // token is the host's only handle on the density: the entry count lives on the device.
    const int64_t per_token = c->cap_nnz_k / (c->cap_tokens > 0 ? c->cap_tokens : 1);
    const bool wide = per_token < 16 && c->n_q_heads <= 32;
    if (c->nnz_block_shift) {
        const KvqSparseBlocked ksp = kvq_blocked_k(c);
        return wide ? launch_qk_sparse_tw<R, 32>(c, ksp, q, scale, scores, ld, s)
                    : launch_qk_sparse_tw<R, 8>(c, ksp, q, scale, scores, ld, s);
    }
    const KvqSparseFlat ksp = kvq_flat_k(c);
    return wide ? launch_qk_sparse_tw<R, 32>(c, ksp, q, scale, scores, ld, s)
                : launch_qk_sparse_tw<R, 8>(c, ksp, q, scale, scores, ld, s);
}

// Attention-sink tokens (paper Sec. 3.5): score of query head blockIdx.y against the fp16 Key of token
// blockIdx.x, overwriting what the quantized kernels wrote there.  One wavefront; lane i owns the
// channel pair (i, i+64).
__global__ __launch_bounds__(64) void kvq_qk_sink(const void *__restrict__ params, int D, int r,
                                                   const uint16_t *__restrict__ sink_k,
                                                   const float *__restrict__ q_rot, float scale,
                                                   float *__restrict__ scores, int64_t ld,
                                                   float *__restrict__ stat_slots, int first_slot)
{
    // stat_slots != null: the token's score also goes into a slot of its own (first_slot + token)
    const KvqParamsView pv = kvq_params_view(params, D);
    const int n = blockIdx.x, qh = blockIdx.y, i = threadIdx.x, kvh = qh / r;
    const float k_lo = kvq_h2f(sink_k[(int64_t)n * D + kvh * 128 + i]);
    const float k_hi = kvq_h2f(sink_k[(int64_t)n * D + kvh * 128 + i + 64]);
    const float qa = q_rot[qh * 128 + i] * scale, qb = q_rot[qh * 128 + i + 64] * scale;
    const float rev = rope_rev((float)n, pv.hdr->rope_vh[i], pv.hdr->rope_vl[i]);
    const float cs = __builtin_amdgcn_cosf(rev), sn = __builtin_amdgcn_sinf(rev);
    float t = (qa * k_lo + qb * k_hi) * cs + (qb * k_lo - qa * k_hi) * sn;
    for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o);
    if (i == 0) {
        scores[(int64_t)qh * ld + n] = t;
        if (stat_slots) stat_slots[(int64_t)qh * KVQ_STAT_SLOTS + first_slot + n] = t;
    }
}

// Store the address of the piece-major kernel's span slots (or null) in its device word and reset the
// slots, on the launch stream: before every launch whose span is taken, and once when the word still
// holds an address and no span is wanted any more.  Part of the timing aid: like the rest of it, not
// meant for calls that overlap.
kvq_status qk3_publish_span(unsigned long long *span, hipStream_t s)
{
    static std::atomic<bool> holds_address[64];            // zero-initialised: the word starts out null
    int dev = 0;
    KVQ_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return span ? KVQ_ERR_UNSUPPORTED : KVQ_OK;
    if (!span && !holds_address[dev].load(std::memory_order_relaxed)) return KVQ_OK;
    static_assert(KVQ_PROFILE_MAX_WGS == 1024, "one thread of the reset kernel per slot pair");
    kvq_qk3_set_span<<<1, KVQ_PROFILE_MAX_WGS, 0, s>>>(span);
    KVQ_HIP_CHECK(hipGetLastError());
    holds_address[dev].store(span != nullptr, std::memory_order_relaxed);
    return KVQ_OK;
}

template <int BITS, int KVH, int RQ, int NT, int PG, int R>
kvq_status launch_qk(const kvq_cache *c, const float *q, float scale, float *scores, int64_t ld, float *stat_slots,
                     int *n_stat, hipStream_t s)
{
    constexpr int QH = KVH * RQ;
    const int D = c->n_kv_heads * KVQ_HEAD_DIM;
    const int64_t L = c->n_tokens_k;
    auto kern = stat_slots ? kvq_qk_kernel<BITS, KVH, RQ, NT, PG, true> : kvq_qk_kernel<BITS, KVH, RQ, NT, PG, false>;
    constexpr bool CAN_SPAN = QH < 8;
    // 3-bit codes, tiles of KVQ_ROPE_STEP tokens: the piece-major kernel (rotary recurrence over TT tiles)
    constexpr bool PIECE_MAJOR = KVQ_QK3_ENABLE && BITS == 3 && NT == KVQ_ROPE_STEP && KVH * KVQ_QK3_TT <= 16;
    // (it addresses the codes with 32-bit offsets)
    const bool piece_major = PIECE_MAJOR && (int64_t)c->n_kv_heads * c->cap_tokens * 16 * BITS < ((int64_t)1 << 32);
    if constexpr (PIECE_MAJOR) {
        if (piece_major)
            kern = stat_slots ? kvq_qk3_kernel<KVH, RQ, KVQ_QK3_TT, KVQ_QK3_PG, true>
                              : kvq_qk3_kernel<KVH, RQ, KVQ_QK3_TT, KVQ_QK3_PG, false>;
    }
    const int groups = c->n_q_heads / QH;
    const int64_t tiles = (L + NT - 1) / NT;
    // about one workgroup per compute unit in total (the tables fill most of a CU's LDS); each
    // workgroup builds its tables once and then streams its share of the tiles
    int64_t gx = kvq_cu_count() / groups;
    if (gx < 1) gx = 1;
    if (gx > 256) gx = 256;          // a head owns 256 statistics slots
    if (gx > tiles) gx = tiles;
    dim3 grid((unsigned)gx, (unsigned)groups);
    KvqProfile &prof = kvq_profile_state();
    unsigned long long *span = CAN_SPAN ? kvq_profile_span_slot(prof, 0, (int64_t)gx * groups) : nullptr;
    if constexpr (PIECE_MAJOR) {
        // the piece-major kernel reads the address of its span slots from device memory: bring that
        // word up to date (null when no spans are taken) before anything of this call is launched
        if (piece_major) {
            kvq_status st = qk3_publish_span(span, s);
            if (st != KVQ_OK) return st;
        } else if (span)
            kern = stat_slots ? kvq_qk_kernel<BITS, KVH, RQ, NT, PG, true, true>
                              : kvq_qk_kernel<BITS, KVH, RQ, NT, PG, false, true>;
    } else if constexpr (CAN_SPAN) {
        if (span)
            kern = stat_slots ? kvq_qk_kernel<BITS, KVH, RQ, NT, PG, true, true>
                              : kvq_qk_kernel<BITS, KVH, RQ, NT, PG, false, true>;
    }
    // the sparse kernel goes first and writes its part of every score; the dense kernel adds its own
    const int sparse_first = !(c->loaded & 2);           // bit 1: thresholds admit no Key outliers
    // bit 2 (set on a copy of the descriptor by kvq_decode_step): the sparse part of every score is in
    // the buffer already, written by the step's first launch
    if (sparse_first && !(c->loaded & KVQ_LOADED_SPARSE_SCORES_DONE)) {
        kvq_status st = launch_qk_sparse<R>(c, q, scale, scores, ld, s);
        if (st != KVQ_OK) return st;
    }
    hipEvent_t *pev = (prof.enabled && prof.use_events) ? prof.ev[0][prof.count[0] % KVQ_PROFILE_RING] : nullptr;
    if (pev) KVQ_HIP_CHECK(hipEventRecord(pev[0], s));
    static_assert(KVQ_STAT_SLOTS >= 256 + KVQ_MAX_SINK, "a slot per workgroup of a head plus the sink tokens");
    const unsigned ns = (unsigned)(c->n_sink < L ? c->n_sink : L);
    kern<<<grid, NT, 0, s>>>(c->params, D, R, c->cap_tokens, L, c->k_codes, q, scale, scores, ld, (int)tiles,
                             sparse_first, stat_slots, (int)ns, span);
    if (pev) KVQ_HIP_CHECK(hipEventRecord(pev[1], s));
    if (prof.enabled) ++prof.count[0];
    if (ns > 0)
        kvq_qk_sink<<<dim3(ns, (unsigned)c->n_q_heads), 64, 0, s>>>(c->params, D, R, c->sink_k, q, scale, scores, ld,
                                                                    stat_slots, (int)gx);
    if (n_stat) *n_stat = (int)gx + (int)ns;
    KVQ_HIP_CHECK(hipGetLastError());
    return KVQ_OK;
}

// Query heads per workgroup: as many as fit the LDS budget (fp32 (A,B) tables: 64 pairs x entries x
// 8 bytes per query head = 8 / 32 / 16 KiB for 2 / 3 / 4 bits).
template <int BITS, int R>
kvq_status dispatch_qk(const kvq_cache *c, const float *q, float scale, float *scores, int64_t ld, float *st,
                       int *n_stat, hipStream_t s)
{
    constexpr int QHMAX = (BITS == 3) ? 4 : 8;
    constexpr int PGD = (BITS == 4) ? 1 : (BITS == 3 ? 4 : 2);
    constexpr int PG = PGD;
    if constexpr (R >= QHMAX) {
        // one KV head per workgroup, QHMAX of its query heads (R / QHMAX workgroups share the KV head)
        return launch_qk<BITS, 1, QHMAX, 1024, PG, R>(c, q, scale, scores, ld, st, n_stat, s);
    } else {
        constexpr int KVH = QHMAX / R;
        // Many heads per workgroup share the rotary sines and cosines but need a long context to keep
        // the chip busy (a workgroup builds its tables once, then takes tiles of 1024 tokens).  With a
        // shorter context that leaves most compute units idle: half as many heads per workgroup and
        // tiles of 512 tokens give four times as many workgroups (two fit a compute unit), one KV head
        // per workgroup 2 * KVH times as many.  The largest grouping that still yields workgroups for
        // five eighths of the compute units is taken.
        const int64_t L = c->n_tokens_k;
        auto workgroups = [&](int kvh, int nt) {
            const int64_t groups = c->n_kv_heads / kvh, tiles = (L + nt - 1) / nt;
            int64_t gx = kvq_cu_count() / groups;
            if (gx < 1) gx = 1;
            if (gx > 256) gx = 256;
            if (gx > tiles) gx = tiles;
            return gx * groups;
        };
        const int64_t enough = (int64_t)kvq_cu_count() * 5 / 8;      // workgroups that keep most of the chip busy
        if (c->n_kv_heads % KVH == 0 && workgroups(KVH, 1024) >= enough)
            return launch_qk<BITS, KVH, R, 1024, PG, R>(c, q, scale, scores, ld, st, n_stat, s);
        if constexpr (KVH >= 4) {
            if (c->n_kv_heads % (KVH / 2) == 0 && workgroups(KVH / 2, 512) >= enough)
                return launch_qk<BITS, KVH / 2, R, 512, PG, R>(c, q, scale, scores, ld, st, n_stat, s);
        }
        // few KV heads or a short context: one KV head per workgroup
        return launch_qk<BITS, 1, R, 512, PG, R>(c, q, scale, scores, ld, st, n_stat, s);
    }
}

template <int BITS>
kvq_status dispatch_qk_r(const kvq_cache *c, const float *q, float scale, float *scores, int64_t ld, float *st,
                         int *n_stat, hipStream_t s)
{
    switch (c->n_q_heads / c->n_kv_heads) {
    case 1: return dispatch_qk<BITS, 1>(c, q, scale, scores, ld, st, n_stat, s);
    case 2: return dispatch_qk<BITS, 2>(c, q, scale, scores, ld, st, n_stat, s);
    case 4: return dispatch_qk<BITS, 4>(c, q, scale, scores, ld, st, n_stat, s);
    case 8: return dispatch_qk<BITS, 8>(c, q, scale, scores, ld, st, n_stat, s);
    default: return KVQ_ERR_UNSUPPORTED;
    }
}

}  // namespace

kvq_status kvq_qk_run(const kvq_cache *cache, const float *d_q_rot, float scale, float *d_scores, int64_t ld_scores,
                      float *stat_slots, int *n_stat, hipStream_t s)
{
    kvq_status st = kvq_check_cache(cache);
    if (st != KVQ_OK) return st;
    if (!cache->loaded) return KVQ_ERR_NOT_LOADED;
    if (!d_q_rot || !d_scores || ((uintptr_t)d_q_rot & 3) || ((uintptr_t)d_scores & 3)) return KVQ_ERR_INVALID_ARG;
    if (ld_scores < cache->n_tokens_k) return KVQ_ERR_INVALID_ARG;
    if (n_stat) *n_stat = 0;
    if (cache->n_tokens_k == 0) return KVQ_OK;
    switch (cache->bits) {
    case 2: return dispatch_qk_r<2>(cache, d_q_rot, scale, d_scores, ld_scores, stat_slots, n_stat, s);
    case 3: return dispatch_qk_r<3>(cache, d_q_rot, scale, d_scores, ld_scores, stat_slots, n_stat, s);
    default: return dispatch_qk_r<4>(cache, d_q_rot, scale, d_scores, ld_scores, stat_slots, n_stat, s);
    }
}

extern "C" kvq_status kvq_qk_matvec(const kvq_cache *cache, const float *d_q_rot, float scale, float *d_scores,
                                    int64_t ld_scores, void *stream)
{
    return kvq_qk_run(cache, d_q_rot, scale, d_scores, ld_scores, nullptr, nullptr, (hipStream_t)stream);
}
