// Attention output against the quantized Value cache (paper Sec. 3.1 per-token Values, App. "Kernel
// Implementation Details"): dense look-up-table mat-vec plus the sparse outlier mat-vec, merged into
// one result.
//
// Design (gfx950).  out[q][c] = sum_n p[q][n] (s_n lut[code_{n,c}] + z_n) + sparse.  The storage format
// keeps the codes of two consecutive tokens of one channel side by side in a 2b-bit field, so the hot
// loop per field is: extract, one LDS gather of the fp16 pair (lut[a], lut[b]) from a layer-wide table,
// two mixed-precision FMAs with the fp32 weights w = p*s of the two tokens.  The table is replicated
// 32 times across LDS banks so gathers never conflict.  Lanes are token pairs, a wavefront owns one
// (query head, 64-channel half) and keeps 64 fp32 accumulators per lane; lanes are summed once at the
// end of the wavefront's token slab.  The zero-point term sum_n p z_n is a per-head scalar.  Sparse
// outliers are handled by a balanced kernel (lanes = outlier entries, fixed-point LDS accumulators);
// all partial results, and the fp16 rows of attention-sink tokens (paper Sec. 3.5) if any, are
// summed in a fixed order by a final small kernel.
#include <utility>
#include "kvq_common.hpp"

#ifndef KVQ_ROTATE_PRIORITY
#define KVQ_ROTATE_PRIORITY 1
#endif

namespace {

constexpr int PV_NT = 256;                 // 4 wavefronts = 4 (query head, half) combinations
constexpr int PV_WAVES = PV_NT / 64;
constexpr int PV_FIELD_GROUP = 8;

struct PvPlan {
    int slabs;              // token slabs of the dense kernel (tiles are split evenly among them)
    int tiles;              // tiles of 128 tokens
    int sslabs;             // workgroups of the sparse kernel
    int swaves;             // its wavefronts per workgroup
    int64_t tokens_per_swave;
    size_t slds;            // its dynamic LDS bytes
};

constexpr int PVS_TW = 16;                // tokens per sub-range of a sparse-kernel wavefront
// row length of the staged probabilities: one token's outliers read the same column of many rows,
// and an odd row length spreads that column over all LDS banks
constexpr int PVS_ROW = PVS_TW + 1;
constexpr int PVS_U = 8;                  // 64-entry batches in flight per wavefront
constexpr int PVS_MAX_SLABS = 512;

__host__ __device__ constexpr int pvs_wave_lds_floats(int n_q_heads)
{
    return n_q_heads * PVS_ROW;                          // the sub-range's probabilities
}

inline PvPlan pv_plan(int64_t L, int n_q_heads)
{
    PvPlan p;
    const int64_t tiles = (L + 127) / 128;
    // aim at ~16 wavefronts per compute unit: CUs * 16 / (2 * Hq) slabs
    int64_t want = ((int64_t)kvq_cu_count() * 16) / (2 * (int64_t)n_q_heads);
    if (want < 1) want = 1;
    if (want > 512) want = 512;
    if (want > tiles) want = tiles;
    p.tiles = (int)tiles;
    p.slabs = (int)want;
    // sparse kernel: LDS holds Hq*128 64-bit accumulators shared by the workgroup plus a private slice
    // per wavefront (two workgroups of 12 wavefronts per CU when they fit in 77 KiB each); the launch
    // fills the chip once (256 CUs, 160 KiB of LDS and 24 wavefronts each, at most PVS_MAX_SLABS
    // workgroups) and every wavefront gets the same number of tokens (a multiple of 8)
    int waves = 12;
    const size_t per_wave = (size_t)pvs_wave_lds_floats(n_q_heads) * 4;
    const size_t shared = (size_t)n_q_heads * (1024 + 8);      // accumulators + per-head score maxima (8 bytes each: alignment)
    while (waves > 1 && shared + waves * per_wave > 78848) waves -= (waves > 4) ? 4 : waves / 2;
    p.swaves = waves;
    p.slds = shared + waves * per_wave;
    int wgs_per_cu = (int)(163840 / p.slds);
    if (wgs_per_cu * waves > 24) wgs_per_cu = 24 / waves;      // six wavefronts per SIMD (register budget)
    if (wgs_per_cu < 1) wgs_per_cu = 1;
    int64_t max_wgs = (int64_t)kvq_cu_count() * wgs_per_cu;
    if (max_wgs > PVS_MAX_SLABS) max_wgs = PVS_MAX_SLABS;
    const int64_t resident = max_wgs * waves;
    int64_t tpw = (L + resident - 1) / resident;
    tpw = (tpw + 7) & ~(int64_t)7;
    if (tpw < 8) tpw = 8;
    const int64_t n_waves = (L + tpw - 1) / tpw;
    p.tokens_per_swave = tpw;
    p.sslabs = (int)((n_waves + waves - 1) / waves);
    if (p.sslabs < 1) p.sslabs = 1;
    return p;
}

template <int FBITS>
__device__ inline uint32_t pv_field_off(const uint32_t *W, int i, uint32_t lane_off)
{
    // (field value * 128) | lane_off : entry e of the replicated table sits at dword e*32 + (lane & 31)
    const int bit = i * FBITS, wi = bit >> 5, sh = bit & 31;
    constexpr uint32_t M = ((1u << FBITS) - 1u) << 7;
    uint32_t x;
    if (sh + FBITS <= 32) {
        if (sh >= 7) x = W[wi] >> (sh - 7);
        else x = W[wi] << (7 - sh);
    } else {
        x = __builtin_amdgcn_alignbit(W[wi + 1], W[wi], sh - 7);   // straddling fields start at bit >= 26
    }
    return kvq_and_or(x, M, lane_off);
}

// One group of PV_FIELD_GROUP fields of a lane's slice.  RG query heads share the fields (grouped-query
// attention): one extraction and one gather per field, two multiply-adds per field and head.
// Accumulator of (head h, field i): acc[h * (64 / RG) + i].
template <int BITS, int RG, int G0>
__device__ __forceinline__ void pv_group(const uint32_t (&W)[4 * BITS / RG], float (&acc)[64], const half2_t *ptab,
                                         uint32_t lane_off, const float (&w0)[RG], const float (&w1)[RG])
{
    constexpr int NF = 64 / RG;
    half2_t t[PV_FIELD_GROUP];
#pragma unroll
    for (int k = 0; k < PV_FIELD_GROUP; ++k) {
        const uint32_t off = pv_field_off<2 * BITS>(W, G0 * PV_FIELD_GROUP + k, lane_off);
        t[k] = *(const half2_t *)((const uint8_t *)ptab + off);
    }
    // the two FMAs of a field depend on each other: issue the group's first halves, then its second
    // halves, so that no instruction waits for the one right before it
#pragma unroll
    for (int h = 0; h < RG; ++h)
#pragma unroll
        for (int k = 0; k < PV_FIELD_GROUP; ++k) {
            float &a = acc[h * NF + G0 * PV_FIELD_GROUP + k];
            a = __builtin_fmaf((float)t[k].x, w0[h], a);
        }
#pragma unroll
    for (int h = 0; h < RG; ++h)
#pragma unroll
        for (int k = 0; k < PV_FIELD_GROUP; ++k) asm volatile("" : "+v"(acc[h * NF + G0 * PV_FIELD_GROUP + k]));
#pragma unroll
    for (int h = 0; h < RG; ++h)
#pragma unroll
        for (int k = 0; k < PV_FIELD_GROUP; ++k) {
            float &a = acc[h * NF + G0 * PV_FIELD_GROUP + k];
            a = __builtin_fmaf((float)t[k].y, w1[h], a);
        }
    // an empty asm that "modifies" the group's accumulators and clobbers memory keeps the groups in
    // order (otherwise every gather of the tile is issued first and register pressure explodes)
#pragma unroll
    for (int h = 0; h < RG; ++h)
#pragma unroll
        for (int k = 0; k < PV_FIELD_GROUP; ++k)
            asm volatile("" : "+v"(acc[h * NF + G0 * PV_FIELD_GROUP + k]) : : "memory");
}

template <int BITS, int RG, int... G>
__device__ __forceinline__ void pv_all_fields(std::integer_sequence<int, G...>, const uint32_t (&W)[4 * BITS / RG],
                                              float (&acc)[64], const half2_t *ptab, uint32_t lane_off,
                                              const float (&w0)[RG], const float (&w1)[RG])
{
    (pv_group<BITS, RG, G>(W, acc, ptab, lane_off, w0, w1), ...);
}

// Dense part.  A wavefront owns one combination of (group of RG query heads that share a KV head,
// 64-channel half, slice of 64/RG channels of that half): its lanes are token pairs and keep the
// RG x 64/RG = 64 accumulators of their pair's fields.  RG = 1: one query head, the whole half.  With
// grouped-query attention RG > 1 heads share every extraction and gather.  grid = (slabs, 2*Hq / 4):
// wavefront w of a workgroup owns combination blockIdx.y*4 + w.  Writes partial[slab][q][128] and
// zpart[slab][q].
// (Four wavefronts per SIMD: the register allocation is held to 128, which every instantiation but
// the 3-bit one for four heads meets without spilling.)
template <int BITS, int RG, bool SPAN = false>
__global__ __launch_bounds__(PV_NT, (BITS == 3 && RG == 4) ? 3 : 4) void kvq_pv_dense(const void *__restrict__ params, int D, int n_kv_heads,
                                                      int n_q_heads, int64_t cap, int64_t L,
                                                      const uint8_t *__restrict__ v_codes,
                                                      const uint16_t *__restrict__ v_sz,
                                                      const float *__restrict__ probs, int64_t ld,
                                                      float *__restrict__ partial, float *__restrict__ zpart,
                                                      int n_tiles, int n_sink,
                                                      const float *__restrict__ stat_slots, int n_stat,
                                                      float *__restrict__ lpart, unsigned long long *span, int n_cu)
{
    if (SPAN) kvq_span_start(span);       // timing-aid instantiation (kvq_profile_*): workgroup start and end times
    // tokens below n_sink are attention-sink tokens kept in fp16: their quantized form gets weight 0
    // here and the reduce kernel adds their fp16 rows.
    // stat_slots != null: `probs` holds raw scores x; a wavefront takes the maximum m of each of its
    // heads' n_stat slots once, weights every token by exp(x - m) as it loads its score, and also writes
    // the sum of these weights over its slab to lpart[slab][q] (the reduce kernel divides by their total)
    constexpr int NE2 = 1 << (2 * BITS);
    constexpr int NF = 64 / RG;                    // fields (channels) per lane and head
    constexpr int ND = 4 * BITS / RG;              // dwords of a chunk that hold them
    static_assert((4 * BITS) % RG == 0 && NF % PV_FIELD_GROUP == 0, "a slice is whole dwords and whole field groups");
    // One array for the replicated pair table (used by the tile loop) and for the lane reduction after
    // it: with the 4-bit table (32 KB) next to the reduction's 17 KB only three workgroups fit a CU.
    constexpr int LDS_WORDS = (NE2 * 32 > PV_WAVES * 64 * 17) ? NE2 * 32 : PV_WAVES * 64 * 17;
    __shared__ __attribute__((aligned(16))) uint32_t lds_words[LDS_WORDS];
    half2_t *ptab = (half2_t *)lds_words;                                 // [NE2 * 32]
    float (*red)[64][17] = (float (*)[64][17])lds_words;                  // [PV_WAVES][64][17]
    const KvqParamsView pv = kvq_params_view(params, D);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int e = tid; e < NE2 * 32; e += PV_NT) {
        const int f = e >> 5;
        ptab[e] = half2_t{(half_t)pv.hdr->lut_v[f & ((1 << BITS) - 1)], (half_t)pv.hdr->lut_v[f >> BITS]};
    }
    __syncthreads();

    const int combo = blockIdx.y * PV_WAVES + wave;
    const bool active = combo < 2 * n_q_heads;
    const int slice = combo % RG, half = (combo / RG) & 1;
    const int q0 = active ? (combo / (2 * RG)) * RG : 0;          // first query head of the group
    const int kvh = q0 / (n_q_heads / n_kv_heads);
    const uint32_t lane_off = (uint32_t)(lane & 31) << 2;
    float m2[RG], lacc[RG], zacc[RG];
#pragma unroll
    for (int h = 0; h < RG; ++h) {
        m2[h] = 0.f; lacc[h] = 0.f; zacc[h] = 0.f;
        if (stat_slots) {
            float m = KVQ_STAT_FLOOR;
            for (int i = lane; i < n_stat; i += 64) m = __builtin_fmaxf(m, stat_slots[(int64_t)(q0 + h) * KVQ_STAT_SLOTS + i]);
            m2[h] = kvq_wave_max(m) * KVQ_LOG2E;
        }
    }

    float acc[64];
#pragma unroll
    for (int j = 0; j < 64; ++j) acc[j] = 0.f;

    const int64_t tile0 = ((int64_t)blockIdx.x * n_tiles) / gridDim.x;
    const int64_t tile1 = ((int64_t)(blockIdx.x + 1) * n_tiles) / gridDim.x;
    // the workgroups that share a compute unit were dispatched n_cu apart; see kvq_set_wave_priority
    const int prio_slot = (int)((blockIdx.y * gridDim.x + blockIdx.x) / (unsigned)n_cu);
    if (active) {
        for (int64_t t = tile0; t < tile1; ++t) {
            if (KVQ_ROTATE_PRIORITY) kvq_set_wave_priority(prio_slot + (int)(t - tile0));
            const int64_t m = t * 64 + lane;                // token pair
            const int64_t n0 = 2 * m;
            if (n0 >= L) continue;
            uint32_t W[ND];
            const uint8_t *p = v_codes + kvq_v_piece0(BITS, cap, m, kvh, half);
            if constexpr (RG == 1) {
#pragma unroll
                for (int j = 0; j < BITS; ++j) {
                    const uint4 v = kvq_load_stream16(p + j * 1024);
                    W[4 * j + 0] = v.x; W[4 * j + 1] = v.y; W[4 * j + 2] = v.z; W[4 * j + 3] = v.w;
                }
            } else {
                // dword d of the chunk sits in 16-byte piece d / 4 (pieces are 1024 bytes apart)
#pragma unroll
                for (int j = 0; j < ND; ++j) {
                    const int d = slice * ND + j;
                    W[j] = *(const uint32_t *)(p + (d >> 2) * 1024 + (d & 3) * 4);
                }
            }
            const uint2 sz = *(const uint2 *)(v_sz + n0 * 2);            // (s0, z0, s1, z1) fp16
            const bool ok0 = n0 >= n_sink, ok1 = n0 + 1 < L && n0 + 1 >= n_sink;   // odd tail: second token absent
            const float s0 = kvq_h2f((uint16_t)(sz.x & 0xFFFFu)), z0 = kvq_h2f((uint16_t)(sz.x >> 16));
            // (scale, zero-point) of an absent second token may be anything, NaN included
            const float s1 = ok1 ? kvq_h2f((uint16_t)(sz.y & 0xFFFFu)) : 0.f, z1 = ok1 ? kvq_h2f((uint16_t)(sz.y >> 16)) : 0.f;
            // The scores (probabilities) are loaded whatever ok0 / ok1 say (the second from an index that
            // always exists), and the empty asm keeps the compiler from moving the loads back under those
            // conditions: a load inside a conditional block is followed by a wait for every load in
            // flight, the tile's codes included, and the tile then costs two or three memory latencies
            // instead of one.
            const int64_t n1 = n0 + 1 < L ? n0 + 1 : n0;
            float pl0[RG], pl1[RG];
#pragma unroll
            for (int h = 0; h < RG; ++h) {
                const float *prow = probs + (int64_t)(q0 + h) * ld;
                pl0[h] = prow[n0];
                pl1[h] = prow[n1];
            }
#pragma unroll
            for (int h = 0; h < RG; ++h) asm volatile("" : "+v"(pl0[h]), "+v"(pl1[h]));
            float w0[RG], w1[RG];
#pragma unroll
            for (int h = 0; h < RG; ++h) {
                float p0 = ok0 ? pl0[h] : 0.f;
                float p1 = ok1 ? pl1[h] : 0.f;
                if (stat_slots) {
                    p0 = ok0 ? kvq_stat_weight(p0, m2[h]) : 0.f;
                    p1 = ok1 ? kvq_stat_weight(p1, m2[h]) : 0.f;
                    lacc[h] += p0 + p1;
                }
                w0[h] = p0 * s0;
                w1[h] = p1 * s1;
                zacc[h] = __builtin_fmaf(p0, z0, zacc[h]);
                zacc[h] = __builtin_fmaf(p1, z1, zacc[h]);
            }
            pv_all_fields<BITS, RG>(std::make_integer_sequence<int, NF / PV_FIELD_GROUP>{}, W, acc, ptab, lane_off, w0, w1);
        }
    }
    if (KVQ_ROTATE_PRIORITY) __builtin_amdgcn_s_setprio(0);
    // sum the 64 lanes: four rounds of 16 accumulators through LDS (over the table, once every
    // wavefront of the workgroup has left the tile loop)
    __syncthreads();
    float outv = 0.f;      // lane l (< 64) ends up with the sum of accumulator l
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
        for (int k = 0; k < 16; ++k) red[wave][lane][k] = acc[r * 16 + k];
        __syncthreads();
        const int col = lane & 15, quarter = lane >> 4;
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j) s += red[wave][quarter * 16 + j][col];
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        if ((lane >> 4) == r) outv = s;          // lanes 16r..16r+15 keep accumulators 16r..16r+15
        __syncthreads();
    }
#pragma unroll
    for (int h = 0; h < RG; ++h) {
        for (int o = 32; o > 0; o >>= 1) zacc[h] += __shfl_xor(zacc[h], o);
        if (stat_slots)
            for (int o = 32; o > 0; o >>= 1) lacc[h] += __shfl_xor(lacc[h], o);
    }
    if (active) {
        // accumulator a = (head a / NF of the group, channel a % NF of the slice)
        const int qh = q0 + lane / NF;
        partial[((int64_t)blockIdx.x * n_q_heads + qh) * 128 + half * 64 + slice * NF + lane % NF] = outv;
        if (half == 0 && slice == 0 && lane == 0) {
#pragma unroll
            for (int h = 0; h < RG; ++h) {
                zpart[(int64_t)blockIdx.x * n_q_heads + q0 + h] = zacc[h];
                if (stat_slots) lpart[(int64_t)blockIdx.x * n_q_heads + q0 + h] = lacc[h];
            }
        }
    }
    if (SPAN) kvq_span_end(span);
}

// Sparse part, balanced (paper App. "Kernel Implementation Details": equal non-zeros per thread):
// lanes are outlier entries, so every lane does the same amount of work whatever the sparsity
// pattern.  A wavefront owns a run of consecutive tokens and walks it PVS_TW tokens at a time on its
// own (no workgroup barrier inside the loop): it stages the sub-range's pointers and probabilities in
// its private LDS slice, finds each entry's token by a binary search over the pointers and adds
// p[q][n] * val to the workgroup's fixed-point LDS accumulators (integer atomics).  The workgroup's
// sums go to the workspace; the reduce kernel adds them up.
// R = query heads per KV head (0: any ratio, looked up at run time); SINK: the cache keeps its first
// n_sink tokens in fp16; FUSED: `probs` holds raw scores, see below (separate instantiations: the
// plain one has no register to spare)
template <int R, bool SINK, bool FUSED, class SP>
__global__ __launch_bounds__(768) __attribute__((amdgpu_waves_per_eu(6, 6)))
void kvq_pv_sparse(int n_kv_heads, int n_q_heads, int64_t L, const uint32_t *__restrict__ v_ptr,
                   const SP vsp, uint32_t nnz_cap,
                   const float *__restrict__ probs, int64_t ld, float *__restrict__ spartial, int64_t tokens_per_wave,
                   int n_sink, const float *__restrict__ stat_slots, int n_stat)
{
    // FUSED: `probs` holds raw scores x; the workgroup takes every head's maximum m over its n_stat
    // slots once and scores become weights exp(x - m) on their way into the wavefront's LDS slice
    extern __shared__ __attribute__((aligned(16))) float dyn[];
    unsigned long long *sacc = (unsigned long long *)dyn;     // [n_q_heads][128] 2^40-scaled sums
    float *sst = (float *)(sacc + n_q_heads * 128);           // [n_q_heads] log2(e) * maximum score (2 floats per head reserved)
    const int tid = threadIdx.x, lane = tid & 63, n_waves = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);           // scalar: loop bounds below are uniform
    float *ps = sst + 2 * n_q_heads + (size_t)wave * pvs_wave_lds_floats(n_q_heads);   // [n_q_heads][PVS_ROW]
    const int r = R ? R : n_q_heads / n_kv_heads;
    for (int j = tid; j < n_q_heads * 128; j += blockDim.x) sacc[j] = 0ull;
    bool cleared = false;      // the barrier after the clearing comes once the first loads are requested
    const int64_t nb = ((int64_t)blockIdx.x * n_waves + wave) * tokens_per_wave;
    int64_t ne = nb + tokens_per_wave;
    if (ne > L) ne = L;
    const int n_cells = n_q_heads * PVS_TW;
    // the run is cut into equal sub-ranges of at most PVS_TW tokens; the pointers of the next one are
    // requested while the current one is processed
    const int run = (nb < ne) ? (int)(ne - nb) : 0, n_sub = (run + PVS_TW - 1) / PVS_TW;
    const int sub_len = n_sub ? (run + n_sub - 1) / n_sub : 0;
    int64_t nc = nb;
    int tc = sub_len;
    uint32_t pw = 0;
    if (tc > 0) pw = v_ptr[nc + (lane < tc ? lane : tc)];
    if (FUSED) {
        // every head's maximum over its slots, four heads per wavefront at a time with their loads
        // requested together (and behind the pointer load above, so that the round trips overlap)
        for (int q0 = 4 * wave; q0 < n_q_heads; q0 += 4 * n_waves) {
            float m[4] = {KVQ_STAT_FLOOR, KVQ_STAT_FLOOR, KVQ_STAT_FLOOR, KVQ_STAT_FLOOR};
            for (int i0 = 0; i0 < n_stat; i0 += 64) {
                const int i = (i0 + lane < n_stat) ? i0 + lane : n_stat - 1;     // a repeated slot does not change a maximum
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int qh = (q0 + k < n_q_heads) ? q0 + k : q0;
                    m[k] = __builtin_fmaxf(m[k], stat_slots[(int64_t)qh * KVQ_STAT_SLOTS + i]);
                }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float w = kvq_wave_max(m[k]) * KVQ_LOG2E;
                if (lane == 0 && q0 + k < n_q_heads) sst[q0 + k] = w;
            }
        }
    }
    while (tc > 0) {
        const int64_t nc_next = nc + tc;
        const int tc_next = (int)((ne - nc_next < sub_len) ? (ne - nc_next) : sub_len);
        // probabilities: cell j = (query head j / 16, token j % 16); loads are straight-line (cells
        // outside the sub-range re-read its first probability and store zero)
        const int t_sink = (SINK && nc < n_sink) ? (int)(n_sink - nc) : 0;    // tokens of this sub-range kept in fp16
        float pr[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int j = lane + 64 * k, qh = j / PVS_TW, t = j % PVS_TW;
            const bool ok = j < n_cells && t < tc;
            const float x = probs[ok ? (int64_t)qh * ld + nc + t : nc];
            pr[k] = (ok && (!SINK || t >= t_sink)) ? x : 0.f;    // sink tokens: weight 0 (kept in fp16)
        }
        const uint32_t e_begin = (uint32_t)__builtin_amdgcn_readfirstlane((int)pw);
        const uint32_t e_end = (uint32_t)__builtin_amdgcn_readlane((int)pw, 63);
        uint32_t chv[PVS_U], vb[PVS_U];
        if (e_begin < e_end) {
            if (e_begin + 64u * PVS_U <= nnz_cap) kvq_sparse_load_batch<false, PVS_U>(vsp, nnz_cap, e_begin, e_end, lane, chv, vb);
            else kvq_sparse_load_batch<true, PVS_U>(vsp, nnz_cap, e_begin, e_end, lane, chv, vb);
        }
        uint32_t pw_next = 0;
        if (tc_next > 0) pw_next = v_ptr[nc_next + (lane < tc_next ? lane : tc_next)];
        if (!cleared) {          // the accumulators are clear and the statistics merged
            __syncthreads();
            cleared = true;
        }
        // (the cells' LDS addresses are recomputed from an opaque copy of the lane number: hoisted
        // out of the loop they would cost eight registers that this kernel does not have)
        int lane_o = lane;
        asm volatile("" : "+v"(lane_o));
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int j = lane_o + 64 * k, qh = j / PVS_TW, t = j % PVS_TW;
            if (j < n_cells) {
                float w = pr[k];
                if (FUSED) {
                    const float e = kvq_stat_weight(w, sst[qh]);
                    w = (t < tc && (!SINK || t >= t_sink)) ? e : 0.f;
                }
                ps[qh * PVS_ROW + t] = w;
            }
        }
        for (int j0 = 64 * 8; j0 < n_cells; j0 += 64) {      // models with more than 32 query heads
            const int j = j0 + lane, qh = j / PVS_TW, t = j % PVS_TW;
            if (j < n_cells) {
                const bool ok = t < tc && (!SINK || t >= t_sink);
                float w = ok ? probs[(int64_t)qh * ld + nc + t] : 0.f;
                if (FUSED && ok) w = kvq_stat_weight(w, sst[qh]);
                ps[qh * PVS_ROW + t] = w;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        int tcur = 0;
        // Every token of a sub-range normally has the same number of outliers (the append keeps
        // 2 * k_side_v per token unless the arrays ran full): entry e then belongs to token
        // (e - e_begin) / per, and the walk over the pointers (kvq_sparse_token, a third of this kernel's
        // time) is not needed.  Checked against the pointers themselves, sub-range by sub-range.
        const float perf = __builtin_truncf(((float)(e_end - e_begin) + 0.5f) * __builtin_amdgcn_rcpf((float)tc));
        const uint32_t per = (uint32_t)perf;
        const bool even = e_end - e_begin < (1u << 22) && per > 0 &&
                          __builtin_amdgcn_ballot_w64(lane <= tc && pw != e_begin + (uint32_t)lane * per) == 0ull;
        const float rper = __builtin_amdgcn_rcpf(perf);
        for (uint32_t eb = e_begin; eb < e_end; eb += 64 * PVS_U) {
            if (eb != e_begin) {                         // (the first batch was requested above)
                if (eb + 64u * PVS_U <= nnz_cap) kvq_sparse_load_batch<false, PVS_U>(vsp, nnz_cap, eb, e_end, lane, chv, vb);
                else kvq_sparse_load_batch<true, PVS_U>(vsp, nnz_cap, eb, e_end, lane, chv, vb);
            }
#pragma unroll
            for (int u = 0; u < PVS_U; ++u) {
                const uint32_t first = eb + 64u * u, e = first + (uint32_t)lane;
                if (first >= e_end) break;
                // ((x + 0.5) / per: the half keeps the quotient's rounding error, 2e-6 at most, away from an integer)
                const int t = even ? (int)(((float)(e - e_begin) + 0.5f) * rper) : kvq_sparse_token(pw, tc, tcur, first, e);
                if (e < e_end) {
                    const uint32_t ch = chv[u];
                    const float v = kvq_h2f((uint16_t)vb[u]);
                    const uint32_t kvh = ch >> 7, c = ch & 127u;
                    for (int j = 0; j < r; ++j) {
                        const uint32_t qh = kvh * r + j;
                        kvq_lds_add_fixed<8>(&sacc[(R == 1) ? ch : qh * 128u + c], ps[qh * PVS_ROW + t] * v);
                    }
                }
            }
        }
        // the next sub-range overwrites ps: order those stores after this sub-range's reads
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        nc = nc_next;
        tc = tc_next;
        pw = pw_next;
    }
    if (!cleared) __syncthreads();       // a wavefront without tokens still meets the workgroup's barrier
    __syncthreads();
    for (int j = tid; j < n_q_heads * 128; j += blockDim.x)
        spartial[(int64_t)blockIdx.x * n_q_heads * 128 + j] = kvq_from_fixed<8>(sacc[j]);
}

// out[q][c] = sum_slabs partial + sum_slabs zpart + sum_sslabs spartial.  Four workgroups per query
// head, each 32 channels x 32 slab groups; every sum is taken in a fixed order.
__global__ __launch_bounds__(1024) void kvq_pv_reduce(int n_q_heads, int slabs, int sslabs,
                                                      const float *__restrict__ partial,
                                                      const float *__restrict__ zpart,
                                                      const float *__restrict__ spartial, float *__restrict__ out,
                                                      int n_sink, int n_kv_heads, const uint16_t *__restrict__ sink_v,
                                                      const float *__restrict__ probs, int64_t ld,
                                                      const float *__restrict__ stat_slots, int n_stat,
                                                      const float *__restrict__ lpart)
{
    // n_sink: attention-sink tokens (already clipped to the tokens present), added from their fp16 rows;
    // stat_slots != null: `probs` holds raw scores, the partial sums are weighted by exp(x - m) (see
    // kvq_pv_dense) and the result is divided by the sum of all weights (lpart, plus the sink tokens')
    __shared__ float red[32][33];
    __shared__ float zred[32], lred[32];
    __shared__ float sm2;
    const int qh = blockIdx.x >> 2, c = (blockIdx.x & 3) * 32 + (threadIdx.x & 31), j = threadIdx.x >> 5;
    if (stat_slots && n_sink > 0 && threadIdx.x < 64) {
        float m = KVQ_STAT_FLOOR;
        for (int i = threadIdx.x; i < n_stat; i += 64) m = __builtin_fmaxf(m, stat_slots[(int64_t)qh * KVQ_STAT_SLOTS + i]);
        m = kvq_wave_max(m) * KVQ_LOG2E;
        if (threadIdx.x == 0) sm2 = m;
    }
    float s = 0.f;
    for (int k0 = j; k0 < slabs; k0 += 256) {          // eight loads in flight per thread
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + 32 * u;
            v[u] = (k < slabs) ? partial[((int64_t)k * n_q_heads + qh) * 128 + c] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (int k0 = j; k0 < sslabs; k0 += 256) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + 32 * u;
            v[u] = (k < sslabs) ? spartial[((int64_t)k * n_q_heads + qh) * 128 + c] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    red[j][threadIdx.x & 31] = s;
    if ((threadIdx.x & 31) == 0) {
        float z = 0.f;
        for (int k = j; k < slabs; k += 32) z += zpart[(int64_t)k * n_q_heads + qh];
        zred[j] = z;
        float l = 0.f;
        if (stat_slots)
            for (int k = j; k < slabs; k += 32) l += lpart[(int64_t)k * n_q_heads + qh];
        lred[j] = l;
    }
    __syncthreads();
    if (j == 0) {
        float t = 0.f, z = 0.f, l = 0.f;
#pragma unroll
        for (int i = 0; i < 32; ++i) { t += red[i][threadIdx.x & 31]; z += zred[i]; l += lred[i]; }
        float sink = 0.f;
        const int kvh = qh / (n_q_heads / n_kv_heads);
        for (int n = 0; n < n_sink; ++n) {
            float w = probs[(int64_t)qh * ld + n];
            if (stat_slots) {
                w = kvq_stat_weight(w, sm2);
                l += w;
            }
            sink = __builtin_fmaf(w, kvq_h2f(sink_v[(int64_t)n * n_kv_heads * 128 + kvh * 128 + c]), sink);
        }
        const float r = t + z + sink;
        out[qh * 128 + c] = stat_slots ? r / l : r;
    }
}

}  // namespace

int64_t kvq_pv_workspace_bytes(int n_q_heads)
{
    // no plan needs more than 512 dense + 512 sparse slabs
    // dense partials, zero-point sums, sparse partials, weight sums (fused call)
    return ((int64_t)512 * n_q_heads * 128 + (int64_t)512 * n_q_heads + (int64_t)512 * n_q_heads * 128 +
            (int64_t)512 * n_q_heads) * 4;
}

extern "C" int64_t kvq_workspace_bytes(const kvq_cache *cache, int32_t max_append)
{
    if (!cache) return 0;
    int64_t a = (int64_t)(max_append > 0 ? max_append : 1) * 4;
    // slab partials of the Value kernels, then the softmax statistics of the fused decode call
    int64_t b = kvq_pv_workspace_bytes(cache->n_q_heads) + (int64_t)cache->n_q_heads * KVQ_STAT_SLOTS * 4;
    int64_t w = a > b ? a : b;
    return (w + 255) & ~(int64_t)255;
}

extern "C" kvq_status kvq_pv_matvec(const kvq_cache *cache, const float *d_probs, int64_t ld_probs, float *d_out,
                                    void *stream)
{
    return kvq_pv_run(cache, d_probs, ld_probs, d_out, nullptr, 0, (hipStream_t)stream);
}

// Launch of the sparse kernel for either layout of the outlier entries.  ri: index of the head ratio
// among {any, 1, 2, 4, 8}.
template <class SP>
static kvq_status pv_launch_sparse(const kvq_cache *cache, const SP vsp, int ri, bool sink, bool fused,
                                   const PvPlan &plan, const float *d_probs, int64_t ld_probs, float *spartial,
                                   const float *stat_slots, int n_stat, hipStream_t s)
{
    using SparseKernel = decltype(&kvq_pv_sparse<0, false, false, SP>);
#define KVQ_PVS_ROW(R) {{kvq_pv_sparse<R, false, false, SP>, kvq_pv_sparse<R, false, true, SP>},       \
                        {kvq_pv_sparse<R, true, false, SP>, kvq_pv_sparse<R, true, true, SP>}}
    static const SparseKernel kernels[5][2][2] = {KVQ_PVS_ROW(0), KVQ_PVS_ROW(1), KVQ_PVS_ROW(2), KVQ_PVS_ROW(4),
                                                  KVQ_PVS_ROW(8)};
#undef KVQ_PVS_ROW
    const SparseKernel sparse = kernels[ri][sink][fused];
    // every instantiation's dynamic-LDS limit is raised once, to the most a plan asks for
    // (initialisation of a function-local static is thread-safe)
    static const hipError_t lds_attr = [] {
        for (auto &a : kernels)
            for (auto &b : a)
                for (SparseKernel k : b) {
                    const hipError_t e = hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, 147456);
                    if (e != hipSuccess) return e;
                }
        return hipSuccess;
    }();
    KVQ_HIP_CHECK(lds_attr);
    if (plan.slds > 147456) return KVQ_ERR_UNSUPPORTED;
    // (Running this kernel on a second stream beside the dense one was tried: its LDS footprint
    // evicts dense workgroups from the CUs and the pair gets slower.)
    if (cache->cap_nnz_v >= ((int64_t)1 << 31)) return KVQ_ERR_UNSUPPORTED;      // byte offsets are 32-bit
    sparse<<<plan.sslabs, 64 * plan.swaves, plan.slds, s>>>(cache->n_kv_heads, cache->n_q_heads, cache->n_tokens_v,
                                                            cache->v_ptr, vsp, (uint32_t)cache->cap_nnz_v, d_probs,
                                                            ld_probs, spartial, plan.tokens_per_swave,
                                                            cache->n_sink, stat_slots, n_stat);
    return KVQ_OK;
}

kvq_status kvq_pv_run(const kvq_cache *cache, const float *d_probs, int64_t ld_probs, float *d_out,
                      const float *stat_slots, int n_stat, hipStream_t s)
{
    kvq_status st = kvq_check_cache(cache);
    if (st != KVQ_OK) return st;
    if (!cache->loaded) return KVQ_ERR_NOT_LOADED;
    if (!d_probs || !d_out || ((uintptr_t)d_probs & 3) || ((uintptr_t)d_out & 3)) return KVQ_ERR_INVALID_ARG;
    const int64_t L = cache->n_tokens_v;
    if (ld_probs < L) return KVQ_ERR_INVALID_ARG;
    const int Hq = cache->n_q_heads, D = cache->n_kv_heads * KVQ_HEAD_DIM;
    if (!cache->workspace || cache->workspace_bytes < kvq_pv_workspace_bytes(Hq)) return KVQ_ERR_CAPACITY;
    const PvPlan plan = (L > 0) ? pv_plan(L, Hq) : PvPlan{0, 0, 0, 0, 0, 0};
    float *partial = (float *)cache->workspace;
    float *zpart = partial + (int64_t)512 * Hq * 128;
    float *spartial = zpart + (int64_t)512 * Hq;
    float *lpart = spartial + (int64_t)512 * Hq * 128;
    if (L > 0) {
        const int r = Hq / cache->n_kv_heads;
        const bool sink = cache->n_sink > 0;
        const int ri = (r == 1) ? 1 : (r == 2) ? 2 : (r == 4) ? 3 : (r == 8) ? 4 : 0;
        const bool fused = stat_slots != nullptr;
        st = cache->nnz_block_shift
                 ? pv_launch_sparse(cache, kvq_blocked_v(cache), ri, sink, fused, plan, d_probs, ld_probs, spartial,
                                    stat_slots, n_stat, s)
                 : pv_launch_sparse(cache, kvq_flat_v(cache), ri, sink, fused, plan, d_probs, ld_probs, spartial,
                                    stat_slots, n_stat, s);
        if (st != KVQ_OK) return st;

        dim3 grid((unsigned)plan.slabs, (unsigned)((2 * Hq + PV_WAVES - 1) / PV_WAVES));
#define LAUNCH_PV(B, G)                                                                                        \
    do {                                                                                                       \
        auto kern = span ? kvq_pv_dense<B, G, true> : kvq_pv_dense<B, G, false>;                               \
        kern<<<grid, PV_NT, 0, s>>>(cache->params, D, cache->n_kv_heads, Hq, cache->cap_tokens, L,             \
                                    cache->v_codes, cache->v_sz, d_probs, ld_probs, partial, zpart,            \
                                    plan.tiles, cache->n_sink, stat_slots, n_stat, lpart, span, kvq_cu_count()); \
    } while (0)
        KvqProfile &prof = kvq_profile_state();
        unsigned long long *span = kvq_profile_span_slot(prof, 1, (int64_t)grid.x * grid.y);
        hipEvent_t *pev = (prof.enabled && prof.use_events) ? prof.ev[1][prof.count[1] % KVQ_PROFILE_RING] : nullptr;
        if (pev) KVQ_HIP_CHECK(hipEventRecord(pev[0], s));
        // query heads of one KV head that a wavefront takes together (they share extraction and gather).
        // When the kernel also turns scores into weights every wavefront that covers a head evaluates
        // that head's exponentials, and grouping multiplies the wavefronts per head: pairs of heads
        // still pay there, fours do not (measured, 32 / 8 heads, 2-bit, 512K tokens: 142 us with two,
        // 155 us with one, 156 us with four heads per wavefront).
        const int rg = stat_slots ? ((r % 2 == 0) ? 2 : 1) : (r % 4 == 0) ? 4 : (r % 2 == 0) ? 2 : 1;
        if (cache->bits == 2) { if (rg == 4) LAUNCH_PV(2, 4); else if (rg == 2) LAUNCH_PV(2, 2); else LAUNCH_PV(2, 1); }
        else if (cache->bits == 3) { if (rg == 4) LAUNCH_PV(3, 4); else if (rg == 2) LAUNCH_PV(3, 2); else LAUNCH_PV(3, 1); }
        else { if (rg == 4) LAUNCH_PV(4, 4); else if (rg == 2) LAUNCH_PV(4, 2); else LAUNCH_PV(4, 1); }
#undef LAUNCH_PV
        if (pev) KVQ_HIP_CHECK(hipEventRecord(pev[1], s));
        if (prof.enabled) ++prof.count[1];
    }
    const int ns = (int)(cache->n_sink < L ? cache->n_sink : L);
    kvq_pv_reduce<<<4 * Hq, 1024, 0, s>>>(Hq, plan.slabs, plan.sslabs, partial, zpart, spartial, d_out, ns,
                                          cache->n_kv_heads, cache->sink_v, d_probs, ld_probs, stat_slots, n_stat, lpart);
    KVQ_HIP_CHECK(hipGetLastError());
    return KVQ_OK;
}
