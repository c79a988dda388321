// Prefill-stage attention over the cache as it stands (gfx950, wave64): the last n_q tokens are the queries, the
// query at absolute position p attends causally to positions 0..p (Eq. 1 under the causal mask).  The paper quantizes
// the cache in the prefill stage too and lets the prompt's own attention read the dequantized K and V (calibration
// design of Section 5.3): quantized tokens enter as X^ = Q(X) s + z (Eq. 2), window tokens as their fp16 values.
//
// This is a dense contraction (4 * D flops per query-token pair), so it runs on the matrix cores:
//   * a work-group of 4 waves owns 128 consecutive queries of one query head, 32 per wave (two 16-query tiles);
//   * the tokens arrive in units of 32 (a packed block or a chunk of the fp16 window).  All 256 threads dequantize
//     the unit once, X^ = fma(code, s, z) in fp32, into LDS as fp16: K^ as [token][channel], V^ transposed as
//     [channel][token].  Dequantized keys are kept as two fp16 numbers (the rounded value and the remainder) and
//     multiplied twice: keys have a few channels of large magnitude, and one fp16 rounding of those, times a large
//     query entry, moves a logit by several 1e-3.  The unit after the current one is fetched into registers while
//     the current one is used;
//   * scores are computed transposed, S^T = K^ Q^T (16x16x32 f16 instructions, tokens along the rows): a lane then
//     holds, for its query, the scores of tokens {4 rq .. 4 rq + 3} and {16 + 4 rq ..}, which is exactly a B operand
//     of O^T += V^T P^T when the A operand (V^T from LDS) lists its tokens in the same order.  The softmax weights
//     therefore go from the accumulator of one product into the operand of the next without leaving the registers;
//   * online softmax in base 2 per query (running maximum shared by the four lanes that hold a query), fp32
//     accumulation, one division at the end.
#include <hip/hip_ext.h>

#include "kvq_internal.h"

namespace kvq {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kQW = 32;                 // queries per wave
constexpr int kQB = kQW * kWaves;       // queries per work-group
constexpr int kKStride = kD + 8;        // halves per K^ row (272 bytes: the 16 rows of a 16-byte read fall on different banks)
constexpr int kVStride = 32 + 8;        // halves per V^ channel row (80 bytes, 16-byte aligned rows)

struct Tiles {
    _Float16 K[32][kKStride];           // K^[token][channel], rounded to fp16
    _Float16 Klo[32][kKStride];         // what the rounding left over (quantized keys only)
    _Float16 Vt[kD][kVStride];          // V^[channel][token]
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Registers of one tensor's unit on its way from memory to LDS.  Quantized: c = codes, s0 / s1 = eight scales (fp32,
// or fp16 packed in s0 alone), z = eight zero-points (fp16); keys grouped per token: s0[0], s0[1] = scales and
// z[0], z[1] = zero-points of the thread's two tokens, as fp32 bits.  fp16 rows (16-bit tensor or window): c and
// s0 = two 16-byte row pieces.
struct Staged { u32x4 c, s0, s1, z; };

__device__ __forceinline__ float half_bits(uint32_t h) { return (float)__builtin_bit_cast(_Float16, (uint16_t)h); }
__device__ __forceinline__ float lo_half(uint32_t w) { return half_bits(w & 0xffffu); }
__device__ __forceinline__ float hi_half(uint32_t w) { return half_bits(w >> 16); }
__device__ __forceinline__ u32x4 ld16(const void *p) { return *reinterpret_cast<const u32x4 *>(p); }

__device__ __forceinline__ uint32_t pack2(float a, float b)
{
    const uint32_t lo = __builtin_bit_cast(uint16_t, (_Float16)a), hi = __builtin_bit_cast(uint16_t, (_Float16)b);
    return lo | (hi << 16);
}
__device__ __forceinline__ u32x4 pack8(const float *x)
{
    return u32x4{pack2(x[0], x[1]), pack2(x[2], x[3]), pack2(x[4], x[5]), pack2(x[6], x[7])};
}

// ---- fp16 rows: thread tid takes 16-byte piece c16 of token t for idx = tid and tid + 256
__device__ __forceinline__ u32x4 load_row_piece(const uint16_t *base, int ring, int pos0, int T, int idx)
{
    const int t = idx >> 4, c16 = idx & 15, pos = pos0 + t;
    u32x4 x = u32x4{0u, 0u, 0u, 0u};                       // tokens past the end read as zero (their weights are zero)
    if (pos < T) x = ld16(base + (size_t)(ring ? pos % ring : pos) * kD + 8 * c16);
    return x;
}

__device__ __forceinline__ void load_rows(const uint16_t *base, int ring, int pos0, int T, int tid, Staged &st)
{
    st.c = load_row_piece(base, ring, pos0, T, tid);
    st.s0 = load_row_piece(base, ring, pos0, T, tid + 256);
    st.s1 = u32x4{0u, 0u, 0u, 0u};
    st.z = u32x4{0u, 0u, 0u, 0u};
}

__device__ __forceinline__ void store_key_rows(Tiles &L, int tid, const Staged &st)
{
    *reinterpret_cast<u32x4 *>(&L.K[tid >> 4][8 * (tid & 15)]) = st.c;
    *reinterpret_cast<u32x4 *>(&L.K[16 + (tid >> 4)][8 * (tid & 15)]) = st.s0;
}

__device__ __forceinline__ void store_value_piece(Tiles &L, int idx, u32x4 x)
{
    const int t = idx >> 4, c16 = idx & 15;
#pragma unroll
    for (int e = 0; e < 8; e++) {
        const uint32_t w = x[e >> 1];
        L.Vt[8 * c16 + e][t] = __builtin_bit_cast(_Float16, (uint16_t)((e & 1) ? w >> 16 : w & 0xffffu));
    }
}

__device__ __forceinline__ void store_value_rows(Tiles &L, int tid, const Staged &st)
{
    store_value_piece(L, tid, st.c);
    store_value_piece(L, tid + 256, st.s0);
}

// ---- metadata: 8 consecutive scales and zero-points starting at index i0 (a multiple of 8)
__device__ __forceinline__ void load_meta8(const float *meta, bool narrow, int i0, Staged &st)
{
    // no branch: with fp16 scales the second load repeats the first (its result is not used)
    const void *p0 = narrow ? static_cast<const void *>(meta_scales16(meta) + i0) : static_cast<const void *>(meta + i0);
    const void *p1 = narrow ? p0 : static_cast<const void *>(meta + i0 + 4);
    st.s0 = ld16(p0);
    st.s1 = ld16(p1);
    st.z = ld16(meta_zeros(meta, narrow) + i0);
}

// the eight scales and zero-points of a staged unit as fp32
__device__ __forceinline__ void unpack_meta8(const Staged &st, bool narrow, float *s, float *z)
{
    if (narrow) {
#pragma unroll
        for (int e = 0; e < 8; e++) s[e] = (e & 1) ? hi_half(st.s0[e >> 1]) : lo_half(st.s0[e >> 1]);
    } else {
#pragma unroll
        for (int e = 0; e < 8; e++) s[e] = __builtin_bit_cast(float, e < 4 ? st.s0[e & 3] : st.s1[e & 3]);
    }
#pragma unroll
    for (int e = 0; e < 8; e++) z[e] = (e & 1) ? hi_half(st.z[e >> 1]) : lo_half(st.z[e >> 1]);
}

// code e (0..7) of the group of eight codes numbered m, from the dwords w0, w1 that hold it
template <int BITS>
__device__ __forceinline__ float code_of(uint32_t w0, uint32_t w1, int m, int e)
{
    if constexpr (BITS == 8) return (float)(((e < 4 ? w0 : w1) >> (8 * (e & 3))) & 255u);
    else if constexpr (BITS == 4) return (float)((w0 >> (4 * ((e >> 1) + 4 * (e & 1)))) & 15u);
    else return (float)((w0 >> (2 * (4 * (m & 1) + (e >> 1) + 8 * (e & 1)))) & 3u);
}

// ---- quantized keys: thread (lane l, channel group cb = tid >> 6) takes the code groups m = cb (token n) and
// m = 4 + cb (token 16 + n), channels 32 cb + 8 kq .. + 7.  c[0], c[1]: dwords of the first group, c[2], c[3]: second.
__device__ __forceinline__ void load_key_codes(const LayerView &lv, size_t blk, int tid, Staged &st)
{
    const int l = tid & 63, cb = tid >> 6, kb = lv.kbits;
    const uint8_t *block = lv.kcode + blk * (size_t)block_code_bytes(kb);
    const bool narrow = lv.narrow != 0;
    const float *meta = lv.kmeta + blk * (size_t)meta_words(narrow);
    // first dword of the two groups: 8 bit -> dwords 2 m, 2 m + 1; 4 bit -> dword m; 2 bit -> dword m / 2
    const int d0 = kb == 8 ? 2 * cb : kb == 4 ? cb : cb >> 1;
    const int d1 = kb == 8 ? 8 + 2 * cb : kb == 4 ? 4 + cb : 2 + (cb >> 1);
    const uint32_t *p0 = reinterpret_cast<const uint32_t *>(block + dword_offset(l, d0));
    const uint32_t *p1 = reinterpret_cast<const uint32_t *>(block + dword_offset(l, d1));
    // the odd dword of an 8-bit group lies in the same 16-byte chunk; narrower codes load the even one twice
    const int odd = kb == 8 ? 1 : 0;
    st.c = u32x4{p0[0], p0[odd], p1[0], p1[odd]};
    if (lv.kpt) {
        // one (s, z) per token and channel group: index 32 * group + token
        const int n = l & 15;
        const int i0 = 32 * cb + n, i1 = i0 + 16;
        st.s0 = u32x4{__builtin_bit_cast(uint32_t, narrow ? half_bits(meta_scales16(meta)[i0]) : meta[i0]),
                      __builtin_bit_cast(uint32_t, narrow ? half_bits(meta_scales16(meta)[i1]) : meta[i1]), 0u, 0u};
        st.s1 = u32x4{0u, 0u, 0u, 0u};
        st.z = u32x4{__builtin_bit_cast(uint32_t, half_bits(meta_zeros(meta, narrow)[i0])),
                     __builtin_bit_cast(uint32_t, half_bits(meta_zeros(meta, narrow)[i1])), 0u, 0u};
    } else {
        load_meta8(meta, narrow, 32 * cb + 8 * (l >> 4), st);
    }
}

template <int BITS>
__device__ __forceinline__ void store_key_codes(const LayerView &lv, Tiles &L, int tid, const Staged &st)
{
    const int l = tid & 63, cb = tid >> 6, n = l & 15, kq = l >> 4;
    const bool kpt = lv.kpt != 0;
    float s[8], z[8];
    unpack_meta8(st, lv.narrow != 0, s, z);                  // (grouped per token: not used)
#pragma unroll
    for (int th = 0; th < 2; th++) {
        const float st_ = __builtin_bit_cast(float, th == 0 ? st.s0[0] : st.s0[1]);
        const float zt_ = __builtin_bit_cast(float, th == 0 ? st.z[0] : st.z[1]);
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; e++)      // m = 4 th + cb: m & 1 == cb & 1
            x[e] = fmaf(code_of<BITS>(st.c[2 * th], st.c[2 * th + 1], cb, e), kpt ? st_ : s[e], kpt ? zt_ : z[e]);
        *reinterpret_cast<u32x4 *>(&L.K[16 * th + n][32 * cb + 8 * kq]) = pack8(x);
#pragma unroll
        for (int e = 0; e < 8; e++) x[e] -= (float)(_Float16)x[e];
        *reinterpret_cast<u32x4 *>(&L.Klo[16 * th + n][32 * cb + 8 * kq]) = pack8(x);
    }
}

// ---- quantized values: thread (lane l, channel group g = tid >> 6) takes the code groups m = 2 g, 2 g + 1
// (channels 16 m + n), tokens 8 kq .. + 7; both share the metadata of group g
__device__ __forceinline__ void load_value_codes(const LayerView &lv, size_t blk, int tid, Staged &st)
{
    const int l = tid & 63, g = tid >> 6, vb = lv.vbits;
    const uint8_t *block = lv.vcode + blk * (size_t)block_code_bytes(vb);
    const bool narrow = lv.narrow != 0;
    const float *meta = lv.vmeta + blk * (size_t)meta_words(narrow);
    // 8 bit: dwords 4 g .. 4 g + 3 (one chunk); 4 bit: dwords 2 g, 2 g + 1; 2 bit: dword g
    const uint32_t *p = reinterpret_cast<const uint32_t *>(block + dword_offset(l, vb == 8 ? 4 * g : vb == 4 ? 2 * g : g));
    // dwords beyond the width's own are loaded from the first again, not from beyond the lane's chunk
    st.c = u32x4{p[0], p[vb >= 4 ? 1 : 0], p[vb == 8 ? 2 : 0], p[vb == 8 ? 3 : 0]};
    load_meta8(meta, narrow, 32 * g + 8 * (l >> 4), st);
}

template <int BITS>
__device__ __forceinline__ void store_value_codes(const LayerView &lv, Tiles &L, int tid, const Staged &st)
{
    const int l = tid & 63, g = tid >> 6, n = l & 15, kq = l >> 4;
    float s[8], z[8];
    unpack_meta8(st, lv.narrow != 0, s, z);
#pragma unroll
    for (int mm = 0; mm < 2; mm++) {
        const uint32_t w0 = BITS == 8 ? st.c[2 * mm] : BITS == 4 ? st.c[mm] : st.c[0];
        const uint32_t w1 = st.c[2 * mm + 1];
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; e++) x[e] = fmaf(code_of<BITS>(w0, w1, mm, e), s[e], z[e]);
        *reinterpret_cast<u32x4 *>(&L.Vt[16 * (2 * g + mm) + n][8 * kq]) = pack8(x);
    }
}

// ---- one unit: memory -> registers, registers -> LDS
struct Stage { Staged k, v; };

__device__ __forceinline__ void load_unit(const PrefillArgs &a, int bh, int u, int T, int tid, Stage &st)
{
    const bool packed = u < a.n_blocks;
    const size_t blk = (size_t)bh * a.NB + u;
    if (packed && a.lv.kbits < 16) load_key_codes(a.lv, blk, tid, st.k);
    else if (packed) load_rows(reinterpret_cast<const uint16_t *>(a.lv.kcode) + (size_t)bh * a.NB * kG * kD, 0, 32 * u, T, tid, st.k);
    else load_rows(a.lv.kres + (size_t)bh * a.RC * kD, a.RC, 32 * u, T, tid, st.k);
    if (packed && a.lv.vbits < 16) load_value_codes(a.lv, blk, tid, st.v);
    else if (packed) load_rows(reinterpret_cast<const uint16_t *>(a.lv.vcode) + (size_t)bh * a.NB * kG * kD, 0, 32 * u, T, tid, st.v);
    else load_rows(a.lv.vres + (size_t)bh * a.RC * kD, a.RC, 32 * u, T, tid, st.v);
}

__device__ __forceinline__ void store_unit(const PrefillArgs &a, int u, int tid, const Stage &st, Tiles &L)
{
    const bool packed = u < a.n_blocks;
    if (packed && a.lv.kbits == 8) store_key_codes<8>(a.lv, L, tid, st.k);
    else if (packed && a.lv.kbits == 4) store_key_codes<4>(a.lv, L, tid, st.k);
    else if (packed && a.lv.kbits == 2) store_key_codes<2>(a.lv, L, tid, st.k);
    else store_key_rows(L, tid, st.k);
    if (packed && a.lv.vbits == 8) store_value_codes<8>(a.lv, L, tid, st.v);
    else if (packed && a.lv.vbits == 4) store_value_codes<4>(a.lv, L, tid, st.v);
    else if (packed && a.lv.vbits == 2) store_value_codes<2>(a.lv, L, tid, st.v);
    else store_value_rows(L, tid, st.v);
}

__device__ __forceinline__ float xor_lanes(float x, int mask) { return __shfl_xor(x, mask, 64); }

__global__ __launch_bounds__(256, 2) void prefill_attention(PrefillArgs a)
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, rq = lane >> 4;
    const int tiles = (a.n_q + kQB - 1) / kQB;
    const int head = blockIdx.x / tiles;                         // b * Hq + query head
    const int tile = tiles - 1 - (int)(blockIdx.x % tiles);      // the longest rows of a head start first
    const int b = head / a.Hq, hq = head % a.Hq;
    const int bh = b * a.Hkv + hq / (a.Hq / a.Hkv);
    const int T = 32 * a.n_blocks + a.n_res;
    const int p0 = T - a.n_q;                                    // absolute position of query 0
    const int i0 = tile * kQB;
    const int ilast = (i0 + kQB < a.n_q ? i0 + kQB : a.n_q) - 1;
    const int units = (p0 + ilast) / 32 + 1;                     // units the work-group walks through
    const int iw = i0 + kQW * wave;                              // first query of this wave
    const int wlast = iw < a.n_q ? (p0 + (iw + kQW - 1 < a.n_q ? iw + kQW - 1 : a.n_q - 1)) / 32 : -1;
    const int wmin = p0 + iw;                                    // units that reach beyond it need the mask

    __shared__ __attribute__((aligned(16))) Tiles L[2];

    // queries of this lane: iq[qt] = iw + 16 qt + n; past the end the last query is repeated and never stored
    int qpos[2];
    half8 Qf[2][4];
#pragma unroll
    for (int qt = 0; qt < 2; qt++) {
        const int i = iw + 16 * qt + n, ic = i < a.n_q ? i : a.n_q - 1;
        qpos[qt] = p0 + ic;
        const uint16_t *row = a.q + ((size_t)head * a.n_q + ic) * kD;
#pragma unroll
        for (int step = 0; step < 4; step++) Qf[qt][step] = *reinterpret_cast<const half8 *>(row + 32 * step + 8 * rq);
    }

    float4v O[8][2];
#pragma unroll
    for (int ct = 0; ct < 8; ct++) { O[ct][0] = float4v{0.0f, 0.0f, 0.0f, 0.0f}; O[ct][1] = float4v{0.0f, 0.0f, 0.0f, 0.0f}; }
    float m[2] = {-INFINITY, -INFINITY}, lsum[2] = {0.0f, 0.0f};

    Stage st;
    load_unit(a, bh, 0, T, tid, st);
    store_unit(a, 0, tid, st, L[0]);
    __syncthreads();
    for (int u = 0; u < units; u++) {
        const Tiles &X = L[u & 1];
        if (u + 1 < units) load_unit(a, bh, u + 1, T, tid, st);          // in flight while this unit is used
        if (u <= wlast) {
            // ---- S^T = K^ Q^T: rows = tokens 16 tt + 4 rq + r, column = query n of tile qt
            float4v S[2][2];
#pragma unroll
            for (int tt = 0; tt < 2; tt++) { S[tt][0] = float4v{0.0f, 0.0f, 0.0f, 0.0f}; S[tt][1] = float4v{0.0f, 0.0f, 0.0f, 0.0f}; }
#pragma unroll
            for (int step = 0; step < 4; step++) {
                const half8 A0 = *reinterpret_cast<const half8 *>(&X.K[n][32 * step + 8 * rq]);
                const half8 A1 = *reinterpret_cast<const half8 *>(&X.K[16 + n][32 * step + 8 * rq]);
#pragma unroll
                for (int qt = 0; qt < 2; qt++) {
                    S[0][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A0, Qf[qt][step], S[0][qt], 0, 0, 0);
                    S[1][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1, Qf[qt][step], S[1][qt], 0, 0, 0);
                }
            }
            if (u < a.n_blocks && a.lv.kbits < 16) {
#pragma unroll
                for (int step = 0; step < 4; step++) {
                    const half8 A0 = *reinterpret_cast<const half8 *>(&X.Klo[n][32 * step + 8 * rq]);
                    const half8 A1 = *reinterpret_cast<const half8 *>(&X.Klo[16 + n][32 * step + 8 * rq]);
#pragma unroll
                    for (int qt = 0; qt < 2; qt++) {
                        S[0][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A0, Qf[qt][step], S[0][qt], 0, 0, 0);
                        S[1][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1, Qf[qt][step], S[1][qt], 0, 0, 0);
                    }
                }
            }
            const bool diag = 32 * u + 31 > wmin;                        // wave-uniform
            half8 P[2];
#pragma unroll
            for (int qt = 0; qt < 2; qt++) {
                float x[8];
#pragma unroll
                for (int e = 0; e < 8; e++) x[e] = S[e >> 2][qt][e & 3] * a.scale_log2e;
                if (diag) {
#pragma unroll
                    for (int e = 0; e < 8; e++)
                        if (32 * u + 16 * (e >> 2) + 4 * rq + (e & 3) > qpos[qt]) x[e] = -INFINITY;
                }
                float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
                mx = fmaxf(mx, xor_lanes(mx, 16));
                mx = fmaxf(mx, xor_lanes(mx, 32));
                // unit 0 holds token 0, which every query sees: the running maximum is finite from the start
                const float mn = fmaxf(m[qt], mx);
                const float alpha = __builtin_amdgcn_exp2f(m[qt] - mn);
                m[qt] = mn;
                float ps = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; e++) { x[e] = __builtin_amdgcn_exp2f(x[e] - mn); ps += x[e]; }
                lsum[qt] = lsum[qt] * alpha + ps;
                if (__any(alpha != 1.0f)) {
#pragma unroll
                    for (int ct = 0; ct < 8; ct++) O[ct][qt] *= alpha;
                }
                P[qt] = half8{(_Float16)x[0], (_Float16)x[1], (_Float16)x[2], (_Float16)x[3],
                              (_Float16)x[4], (_Float16)x[5], (_Float16)x[6], (_Float16)x[7]};
            }
            // ---- O^T += V^T P^T: rows = channels 16 ct + 4 rq + r; both operands list the tokens as
            // {4 rq .. 4 rq + 3, 16 + 4 rq .. 16 + 4 rq + 3}
#pragma unroll
            for (int ct = 0; ct < 8; ct++) {
                const half4 v0 = *reinterpret_cast<const half4 *>(&X.Vt[16 * ct + n][4 * rq]);
                const half4 v1 = *reinterpret_cast<const half4 *>(&X.Vt[16 * ct + n][16 + 4 * rq]);
                const half8 A = half8{v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                O[ct][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A, P[0], O[ct][0], 0, 0, 0);
                O[ct][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A, P[1], O[ct][1], 0, 0, 0);
            }
        }
        if (u + 1 < units) store_unit(a, u + 1, tid, st, L[(u + 1) & 1]);
        __syncthreads();
    }

#pragma unroll
    for (int qt = 0; qt < 2; qt++) {
        float l = lsum[qt];
        l += xor_lanes(l, 16);
        l += xor_lanes(l, 32);
        const int i = iw + 16 * qt + n;
        if (i < a.n_q) {
            const float inv = 1.0f / l;
            uint16_t *row = a.out + ((size_t)head * a.n_q + i) * kD;
#pragma unroll
            for (int ct = 0; ct < 8; ct++)
                *reinterpret_cast<uint2 *>(row + 16 * ct + 4 * rq) =
                    make_uint2(pack2(O[ct][qt][0] * inv, O[ct][qt][1] * inv), pack2(O[ct][qt][2] * inv, O[ct][qt][3] * inv));
        }
    }
}

}  // namespace

hipError_t launch_prefill_attention(const PrefillArgs &a, hipStream_t s, hipEvent_t ev_begin, hipEvent_t ev_end)
{
    const long long tiles = (a.n_q + kQB - 1) / kQB;
    const long long groups = tiles * a.B * a.Hq;
    if (groups < 1 || groups > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const dim3 grid((unsigned)groups), block(256);
    if (ev_begin && ev_end) hipExtLaunchKernelGGL(prefill_attention, grid, block, 0, s, ev_begin, ev_end, 0, a);
    else hipLaunchKernelGGL(prefill_attention, grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace kvq
