// Prefill-stage attention over the cache as it stands (gfx950, wave64): the last n_q tokens are the queries, the
// query at absolute position p attends causally to positions 0..p (Eq. 1 under the causal mask).  The paper quantizes
// the cache in the prefill stage too and lets the prompt's own attention read the dequantized K and V (calibration
// design of Section 5.3): quantized tokens enter as X^ = Q(X) s + z (Eq. 2), window tokens as their fp16 values.
//
// This is a dense contraction (4 * D flops per query-token pair), so it runs on the matrix cores, in two passes over a
// chunk of (batch, kv head) caches at a time, behind one small kernel per call:
//   0. prefill_select (keys quantized per channel): the low parts of the keys (below) cost a third of the matrix
//      instructions, and they matter in the channels where keys and queries are large.  Per cache, from the stored
//      scales and zero-points and a sample of the queries, the kernel (a) finds every channel's centre, which pass 1
//      takes off the dequantized keys: a constant per channel moves all scores of a query alike and the softmax does
//      not see it, so an offset that a channel's keys share no longer costs fp16 precision (the window's fp16 rows keep
//      theirs; their scores are lowered by q . centre instead); (b) picks the 32 channels where one fp16 rounding of
//      the centred keys moves the logits most and checks that in all the others together it moves them by less than
//      the fp16 softmax weights are rounded by anyway; then only those 32 keep their low parts (one batch of score
//      products instead of four), otherwise all 128 do.
//   1. prefill_dequantize: every packed unit (32 tokens) of the chunk is dequantized once, X^ = fma(code, s, z) in
//      fp32, into a scratch area as fp16, in the layout the attention kernel keeps a unit in LDS: K^ as
//      [token][channel], V^ transposed as [channel][token].  Dequantized keys are multiplied by the softmax constant
//      log2(e) / sqrt(D) in fp32 (the score products then come out in the exponent's units) and kept as two fp16
//      numbers (the rounded value and the remainder), which are multiplied twice: keys have a few channels of large
//      magnitude, and one fp16 rounding of those, times a large query entry, moves a logit by several 1e-3.
//      Dequantizing inside the attention
//      kernel instead repeats this work for every query head of the group and every query tile (256 times per unit at
//      8192 queries) and made that kernel bound by its vector instructions.
//   2. prefill_attention: a work-group of 8 waves owns 256 consecutive queries of one query head, 32 per wave (two
//      16-query tiles).  The units are fetched from the scratch area straight into LDS (fp16 window chunks: from the
//      ring, through registers), five tile buffers, two units per barrier, so that the score products of the next
//      unit can be issued next to the softmax weights of the current one.  Scores are computed transposed, S^T = K^ Q^T
//      (16x16x32 f16 instructions, tokens along the rows): a lane then holds, for its query, the scores of tokens
//      {4 rq .. 4 rq + 3} and {16 + 4 rq ..}, which is exactly a B operand of O^T += V^T P^T when the A operand (V^T
//      from LDS) lists its tokens in the same order.  The softmax weights therefore go from the accumulator of one
//      product into the operand of the next without leaving the registers.  Online softmax in base 2 per query (the
//      reference is shared by the four lanes that hold a query and only moves when a score exceeds it by more than 8
//      in the exponent; the score products of quantized keys start from minus the reference, so that in the common
//      case their results are the exponents themselves), fp32 accumulation, one division at the end.
#include <hip/hip_ext.h>

#include <type_traits>

#include "kvq_internal.h"

namespace kvq {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kWaves = 8;                // waves of an attention work-group
constexpr int kStagers = 4;              // waves that turn a unit into tiles (256 threads: the thread -> code maps below)
constexpr int kQT = 2;                   // tiles of 16 queries per wave
constexpr int kQW = 16 * kQT;            // queries per wave
constexpr int kQB = kQW * kWaves;       // queries per work-group
constexpr int kKStride = kD + 16;       // halves per K^ row: 288 bytes.  Measured with a probe kernel: the 16-byte operand reads of a wave
                                        // (16 rows x 4 pieces) take 3.9 LDS cycles at this stride, like a linear read; 7.8 + 3.9 conflict cycles at 272
constexpr int kVStride = 32 + 4;        // halves per V^ channel row (72 bytes = 18 banks: the 16 rows of an 8-byte read fall on different banks)

struct Tiles {
    _Float16 K[32][kKStride];           // K^[token][channel], rounded to fp16
    _Float16 Klo[32][kKStride];         // what the rounding left over (quantized keys only)
    _Float16 Vt[kD][kVStride];          // V^[channel][token]
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Which key channels of a (batch, kv head) cache keep the remainders of their fp16 rounding (prefill_select).  In the
// compact form only the 32 selected channels do, and their remainders are stored as a tile [token][slot] of
// kLoStride halves per row at the place of Tiles::Klo (the first 2.5 KiB of it): one batch of the score products
// instead of four.
struct Select {
    uint8_t pos[kD];          // slot (0..31) of a channel's remainders in the compact tile, 255 = none kept
    uint8_t chan[32];         // the channel of a slot
    uint32_t compact;         // 0: every channel keeps its remainder (Tiles::Klo as declared)
    uint8_t pad[92];
    float centre[kD];         // per channel: subtracted from every dequantized key of the cache before it is rounded
};
static_assert(sizeof(Select) == 768, "one record per cache");
constexpr int kLoStride = 32 + 8;       // halves per row of the compact tile: 80 bytes = 20 banks, the 16-byte reads of a wave
                                        // (16 rows x 4 pieces) fall on every bank exactly four times
constexpr int kLoPieces = 3;            // KiB of the compact tile that are fetched (32 rows x 80 bytes = 2.5 KiB)
// how the keys' low parts enter the attention kernel
constexpr int kLoNone = 0, kLoAll = 1, kLoCompact = 2;

// Metadata of the unit being dequantized (in LDS), one slab per wave (wave w dequantizes channel group w of the keys and of the
// values, so it needs 32 scales and 32 zero-points of each tensor and nobody else's): written and read by the same
// wave, no work-group barrier in between.
struct MetaSlab {
    uint32_t ks[32];     // key scales (fp32, or 32 fp16 numbers in the first 16 dwords)
    uint16_t kz[32];     // key zero-points
    uint32_t vs[32];     // value scales
    uint16_t vz[32];     // value zero-points
};

// Registers of a unit on its way from the packed cache to the tiles.  Quantized tensor: k0 / v0 = the dwords of the thread's two code
// groups; fp16 rows (16-bit tensor or window): k0, k1 / v0, v1 = two 16-byte row pieces.  m = this lane's 16-byte
// piece of the wave's metadata (lanes 0..23).
struct Stage { u32x4 k0, k1, v0, v1, m; };

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float half_bits(uint32_t h) { return (float)__builtin_bit_cast(_Float16, (uint16_t)h); }
__device__ __forceinline__ u32x4 ld16(const void *p) { return *reinterpret_cast<const u32x4 *>(p); }
__device__ __forceinline__ u32x4 zero4() { return u32x4{0u, 0u, 0u, 0u}; }

__device__ __forceinline__ uint32_t pack2(float a, float b)
{
    const uint32_t lo = __builtin_bit_cast(uint16_t, (_Float16)a), hi = __builtin_bit_cast(uint16_t, (_Float16)b);
    return lo | (hi << 16);
}
__device__ __forceinline__ u32x4 pack8(const float *x)
{
    return u32x4{pack2(x[0], x[1]), pack2(x[2], x[3]), pack2(x[4], x[5]), pack2(x[6], x[7])};
}

// ---- fp16 rows: thread tid takes 16-byte piece c16 of token t for idx = tid and tid + 256.  A token past the end reads
// the last one instead; it is zeroed on its way to LDS (an operation on the loaded value right here would make the
// wave wait for the load where it is issued).
__device__ __forceinline__ u32x4 load_row_piece(const uint16_t *base, int ring, int pos0, int T, int idx)
{
    const int t = idx >> 4, c16 = idx & 15, pos = pos0 + t, pc = pos < T ? pos : T - 1;
    return ld16(base + (size_t)(ring ? pc % ring : pc) * kD + 8 * c16);
}

// tokens past the end count as zero (their weights are zero)
__device__ __forceinline__ u32x4 live_piece(u32x4 x, int pos0, int T, int idx)
{
    const bool live = pos0 + (idx >> 4) < T;
    return u32x4{live ? x[0] : 0u, live ? x[1] : 0u, live ? x[2] : 0u, live ? x[3] : 0u};
}

__device__ __forceinline__ void store_key_rows(Tiles &L, int tid, u32x4 r0, u32x4 r1)
{
    *reinterpret_cast<u32x4 *>(&L.K[tid >> 4][8 * (tid & 15)]) = r0;
    *reinterpret_cast<u32x4 *>(&L.K[16 + (tid >> 4)][8 * (tid & 15)]) = r1;
}

// value rows are staged with the token index fastest across the lanes (piece idx: token idx & 31, 16-byte piece
// idx >> 5): the transposed 2-byte writes of a wave then fall on consecutive addresses instead of on two banks
__device__ __forceinline__ u32x4 load_value_row_piece(const uint16_t *base, int ring, int pos0, int T, int idx)
{
    const int t = idx & 31, c16 = idx >> 5, pos = pos0 + t, pc = pos < T ? pos : T - 1;
    return ld16(base + (size_t)(ring ? pc % ring : pc) * kD + 8 * c16);
}

__device__ __forceinline__ void store_value_piece(Tiles &L, int idx, u32x4 x, int pos0, int T)
{
    const int t = idx & 31, c16 = idx >> 5;
    const bool live = pos0 + t < T;                        // tokens past the end count as zero
#pragma unroll
    for (int e = 0; e < 8; e++) {
        const uint32_t w = x[e >> 1];
        L.Vt[8 * c16 + e][t] = __builtin_bit_cast(_Float16, (uint16_t)(live ? ((e & 1) ? w >> 16 : w & 0xffffu) : 0u));
    }
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
// m = 4 + cb (token 16 + n), channels 32 cb + 8 kq .. + 7.  Returned: [0], [1] dwords of the first group, [2], [3] of
// the second.  Always four loads (codes narrower than 8 bits load their one dword twice): the number of loads in
// flight does not depend on the bit width.
__device__ __forceinline__ u32x4 load_key_codes(const LayerView &lv, size_t blk, int tid)
{
    const int l = tid & 63, cb = tid >> 6, kb = lv.kbits;
    const uint8_t *block = lv.kcode + blk * (size_t)block_code_bytes(kb);
    // first dword of the two groups: 8 bit -> dwords 2 m, 2 m + 1 (same 16-byte chunk); 4 bit -> dword m; 2 bit -> dword m / 2
    const int d0 = kb == 8 ? 2 * cb : kb == 4 ? cb : cb >> 1;
    const int d1 = kb == 8 ? 8 + 2 * cb : kb == 4 ? 4 + cb : 2 + (cb >> 1);
    const uint32_t *p0 = reinterpret_cast<const uint32_t *>(block + dword_offset(l, d0));
    const uint32_t *p1 = reinterpret_cast<const uint32_t *>(block + dword_offset(l, d1));
    const int odd = kb == 8 ? 1 : 0;
    return u32x4{p0[0], p0[odd], p1[0], p1[odd]};
}

// ---- quantized values: thread (lane l, channel group g = tid >> 6) takes the code groups m = 2 g, 2 g + 1
// (channels 16 m + n), tokens 8 kq .. + 7.  8 bit: dwords 4 g .. 4 g + 3 (one chunk); 4 bit: dwords 2 g, 2 g + 1;
// 2 bit: dword g; dwords beyond the width's own are loaded from the first again.
__device__ __forceinline__ u32x4 load_value_codes(const LayerView &lv, size_t blk, int tid)
{
    const int l = tid & 63, g = tid >> 6, vb = lv.vbits;
    const uint8_t *block = lv.vcode + blk * (size_t)block_code_bytes(vb);
    const uint32_t *p = reinterpret_cast<const uint32_t *>(block + dword_offset(l, vb == 8 ? 4 * g : vb == 4 ? 2 * g : g));
    return u32x4{p[0], p[vb >= 4 ? 1 : 0], p[vb == 8 ? 2 : 0], p[vb == 8 ? 3 : 0]};
}

// ---- this lane's piece of the wave's metadata: lanes 0..11 keys, 12..23 values; of each, pieces 0..7 are the 32
// scales of channel group w (fp16 scales: pieces 0..3 only) and 8..11 the 32 zero-points
__device__ __forceinline__ u32x4 load_meta_piece(const LayerView &lv, size_t blk, int wave, int lane, bool kq, bool vq)
{
    const bool narrow = lv.narrow != 0;
    const int tensor = lane >= 12 ? 1 : 0, j = lane - 12 * tensor;
    const float *meta = (tensor ? lv.vmeta : lv.kmeta) + blk * (size_t)meta_words(narrow);
    const bool wanted = lane < 24 && (tensor ? vq : kq) && !(narrow && j >= 4 && j < 8);
    const uint8_t *src = j < 8 ? reinterpret_cast<const uint8_t *>(meta) + (narrow ? 64 : 128) * wave + 16 * j
                               : reinterpret_cast<const uint8_t *>(meta_zeros(meta, narrow)) + 64 * wave + 16 * (j - 8);
    // lanes with nothing to fetch read the start of the key codes instead (the result is not used): one load per unit
    // on every path
    return ld16(wanted ? src : lv.kcode);
}

__device__ __forceinline__ void store_meta_piece(MetaSlab &M, int lane, u32x4 x)
{
    if (lane < 24) {
        const int tensor = lane >= 12 ? 1 : 0, j = lane - 12 * tensor;
        uint32_t *dst = j < 8 ? (tensor ? M.vs : M.ks) + 4 * j : reinterpret_cast<uint32_t *>(tensor ? M.vz : M.kz) + 4 * (j - 8);
        *reinterpret_cast<u32x4 *>(dst) = x;
    }
}

// eight consecutive scales / zero-points of a slab, starting at index i0 (a multiple of 8), as fp32
__device__ __forceinline__ void slab_meta8(const uint32_t *scales, const uint16_t *zeros, bool narrow, int i0, float *s, float *z)
{
    if (narrow) {
        const u32x4 a = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(scales) + i0);
#pragma unroll
        for (int e = 0; e < 8; e++) s[e] = half_bits((e & 1) ? a[e >> 1] >> 16 : a[e >> 1] & 0xffffu);
    } else {
        const u32x4 a = *reinterpret_cast<const u32x4 *>(scales + i0), b = *reinterpret_cast<const u32x4 *>(scales + i0 + 4);
#pragma unroll
        for (int e = 0; e < 8; e++) s[e] = __builtin_bit_cast(float, e < 4 ? a[e & 3] : b[e & 3]);
    }
    const u32x4 c = *reinterpret_cast<const u32x4 *>(zeros + i0);
#pragma unroll
    for (int e = 0; e < 8; e++) z[e] = half_bits((e & 1) ? c[e >> 1] >> 16 : c[e >> 1] & 0xffffu);
}

// kscale: the softmax constant log2(e) / sqrt(D), multiplied into the dequantized keys in fp32 before they are split
// into two fp16 numbers: the attention kernel's score products then come out in the exponent's units.
// rec: the cache's selection record or null; compact: its low parts go into the compact tile
template <int BITS, bool KPT>
__device__ __forceinline__ void store_key_codes(const LayerView &lv, Tiles &L, const MetaSlab &M, int tid, u32x4 c, float kscale,
                                                const Select *rec, bool compact)
{
    const int l = tid & 63, cb = tid >> 6, n = l & 15, kq = l >> 4;
    const bool narrow = lv.narrow != 0;
    float s[8], z[8];
    if constexpr (!KPT) {
        slab_meta8(M.ks, M.kz, narrow, 8 * kq, s, z);                          // one (s, z) per channel
        if (rec) {
            // the channel's centre goes off with the zero-point: a constant per channel moves every score of a query
            // alike, which the softmax does not see (window tokens: see attend)
            const float4 c0 = *reinterpret_cast<const float4 *>(&rec->centre[32 * cb + 8 * kq]);
            const float4 c1 = *reinterpret_cast<const float4 *>(&rec->centre[32 * cb + 8 * kq + 4]);
            z[0] -= c0.x; z[1] -= c0.y; z[2] -= c0.z; z[3] -= c0.w;
            z[4] -= c1.x; z[5] -= c1.y; z[6] -= c1.z; z[7] -= c1.w;
        }
    }
#pragma unroll
    for (int th = 0; th < 2; th++) {
        const int t = 16 * th + n;
        if constexpr (KPT) {
            // grouped per token: one (s, z) for this token and channel group
            const float st_ = narrow ? half_bits(reinterpret_cast<const uint16_t *>(M.ks)[t]) : __builtin_bit_cast(float, M.ks[t]);
            const float zt_ = half_bits(M.kz[t]);
#pragma unroll
            for (int e = 0; e < 8; e++) { s[e] = st_; z[e] = zt_; }
        }
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; e++)      // m = 4 th + cb: m & 1 == cb & 1
            x[e] = fmaf(code_of<BITS>(th == 0 ? c[0] : c[2], th == 0 ? c[1] : c[3], cb, e), s[e], z[e]) * kscale;
        *reinterpret_cast<u32x4 *>(&L.K[t][32 * cb + 8 * kq]) = pack8(x);
#pragma unroll
        for (int e = 0; e < 8; e++) x[e] -= (float)(_Float16)x[e];
        if (compact) {
            const u32x2 pw = *reinterpret_cast<const u32x2 *>(&rec->pos[32 * cb + 8 * kq]);
            _Float16 *row = &L.Klo[0][0] + t * kLoStride;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const uint32_t slot = ((e < 4 ? pw[0] : pw[1]) >> (8 * (e & 3))) & 255u;
                if (slot < 32u) row[slot] = (_Float16)x[e];
            }
        } else {
            *reinterpret_cast<u32x4 *>(&L.Klo[t][32 * cb + 8 * kq]) = pack8(x);
        }
    }
}

template <int BITS>
__device__ __forceinline__ void store_value_codes(const LayerView &lv, Tiles &L, const MetaSlab &M, int tid, u32x4 c)
{
    const int l = tid & 63, g = tid >> 6, n = l & 15, kq = l >> 4;
    float s[8], z[8];
    slab_meta8(M.vs, M.vz, lv.narrow != 0, 8 * kq, s, z);
#pragma unroll
    for (int mm = 0; mm < 2; mm++) {
        const uint32_t w0 = BITS == 8 ? (mm == 0 ? c[0] : c[2]) : BITS == 4 ? (mm == 0 ? c[0] : c[1]) : c[0];
        const uint32_t w1 = mm == 0 ? c[1] : c[3];
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; e++) x[e] = fmaf(code_of<BITS>(w0, w1, mm, e), s[e], z[e]);
        const u32x4 h = pack8(x);                          // rows are 8-byte aligned only
        uint2 *dst = reinterpret_cast<uint2 *>(&L.Vt[16 * (2 * g + mm) + n][8 * kq]);
        dst[0] = make_uint2(h[0], h[1]);
        dst[1] = make_uint2(h[2], h[3]);
    }
}

// ---- one packed unit: packed cache -> registers, registers -> tiles (LDS or the scratch area: the stores below only
// see a reference).  KQ / VQ: the layer's keys / values are quantized (else fp16 rows in the code area).
template <bool KQ, bool VQ>
__device__ __forceinline__ void load_packed(const PrefillArgs &a, int bh, int u, int T, int tid, Stage &st)
{
    const size_t blk = (size_t)bh * a.NB + u;
    if constexpr (KQ) {
        st.k0 = load_key_codes(a.lv, blk, tid);
        st.k1 = zero4();
    } else {
        const uint16_t *rows = reinterpret_cast<const uint16_t *>(a.lv.kcode) + (size_t)bh * a.NB * kG * kD;
        st.k0 = load_row_piece(rows, 0, 32 * u, T, tid);
        st.k1 = load_row_piece(rows, 0, 32 * u, T, tid + 256);
    }
    if constexpr (VQ) {
        st.v0 = load_value_codes(a.lv, blk, tid);
        st.v1 = zero4();
    } else {
        const uint16_t *rows = reinterpret_cast<const uint16_t *>(a.lv.vcode) + (size_t)bh * a.NB * kG * kD;
        st.v0 = load_value_row_piece(rows, 0, 32 * u, T, tid);
        st.v1 = load_value_row_piece(rows, 0, 32 * u, T, tid + 256);
    }
    if constexpr (KQ || VQ) st.m = load_meta_piece(a.lv, blk, tid >> 6, tid & 63, KQ, VQ);
    else st.m = zero4();
}

template <bool KQ, bool VQ>
__device__ __forceinline__ void store_packed(const PrefillArgs &a, int tid, const Stage &st, Tiles &L, MetaSlab &M, const Select *rec)
{
    const bool compact = rec && rec->compact != 0;
    if constexpr (KQ || VQ) {
        wave_lds_sync();                                   // the slab's readers of the unit before are done
        store_meta_piece(M, tid & 63, st.m);
        wave_lds_sync();
    }
    if constexpr (KQ) {
        if (a.lv.kpt) {
            if (a.lv.kbits == 8) store_key_codes<8, true>(a.lv, L, M, tid, st.k0, a.scale_log2e, rec, compact);
            else if (a.lv.kbits == 4) store_key_codes<4, true>(a.lv, L, M, tid, st.k0, a.scale_log2e, rec, compact);
            else store_key_codes<2, true>(a.lv, L, M, tid, st.k0, a.scale_log2e, rec, compact);
        } else {
            if (a.lv.kbits == 8) store_key_codes<8, false>(a.lv, L, M, tid, st.k0, a.scale_log2e, rec, compact);
            else if (a.lv.kbits == 4) store_key_codes<4, false>(a.lv, L, M, tid, st.k0, a.scale_log2e, rec, compact);
            else store_key_codes<2, false>(a.lv, L, M, tid, st.k0, a.scale_log2e, rec, compact);
        }
    } else {
        store_key_rows(L, tid, st.k0, st.k1);
    }
    if constexpr (VQ) {
        if (a.lv.vbits == 8) store_value_codes<8>(a.lv, L, M, tid, st.v0);
        else if (a.lv.vbits == 4) store_value_codes<4>(a.lv, L, M, tid, st.v0);
        else store_value_codes<2>(a.lv, L, M, tid, st.v0);
    } else {
        store_value_piece(L, tid, st.v0, 0, 32);
        store_value_piece(L, tid + 256, st.v1, 0, 32);
    }
}

// ---- one chunk of the fp16 window, ring -> LDS tiles (at most two chunks per work-group: staged without overlap)
__device__ __forceinline__ void stage_window(const PrefillArgs &a, int bh, int u, int T, int tid, Tiles &L)
{
    const uint16_t *krows = a.lv.kres + (size_t)bh * a.RC * kD, *vrows = a.lv.vres + (size_t)bh * a.RC * kD;
    const u32x4 k0 = load_row_piece(krows, a.RC, 32 * u, T, tid), k1 = load_row_piece(krows, a.RC, 32 * u, T, tid + 256);
    const u32x4 v0 = load_value_row_piece(vrows, a.RC, 32 * u, T, tid), v1 = load_value_row_piece(vrows, a.RC, 32 * u, T, tid + 256);
    store_key_rows(L, tid, live_piece(k0, 32 * u, T, tid), live_piece(k1, 32 * u, T, tid + 256));
    store_value_piece(L, tid, v0, 32 * u, T);
    store_value_piece(L, tid + 256, v1, 32 * u, T);
}

__device__ __forceinline__ float xor_lanes(float x, int mask) { return __shfl_xor(x, mask, 64); }

// ---- the three phases of one unit (32 tokens, in X) against the 32 queries of a wave

// S^T = K^ Q^T: rows = tokens 16 tt + 4 rq + r, column = query n of tile qt.  KLO: quantized keys, whose fp16 rounding
// remainders are multiplied as well.
// the A operand of the output product for channel tile ct: V^T rows 16 ct + n, tokens {4 rq .. + 3, 16 + 4 rq .. + 3}
__device__ __forceinline__ half8 value_operand(const Tiles &X, int ct, int n, int rq)
{
    const half4 v0 = *reinterpret_cast<const half4 *>(&X.Vt[16 * ct + n][4 * rq]);
    const half4 v1 = *reinterpret_cast<const half4 *>(&X.Vt[16 * ct + n][16 + 4 * rq]);
    return half8{v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
}

struct NoSlice { __device__ __forceinline__ void operator()(int) const {} };

// batches of score products per unit: four for the keys' 128 channels, then those of the low parts
template <int LO> constexpr int score_batches() { return LO == kLoAll ? 8 : LO == kLoCompact ? 5 : 4; }

// LO: how the low parts of quantized keys come (none: fp16 rows; all channels: Tiles::Klo; compact: the tile of the 32
// selected channels, against Qlo = the queries' values at those channels).
template <int LO, class Slice = NoSlice>
__device__ __forceinline__ void score_unit(const Tiles &X, const half8 (&Qf)[kQT][4], const half8 (&Qlo)[kQT], float4v (&S)[2][kQT],
                                           int n, int rq, const float4v (&init)[kQT], const Tiles *Xv = nullptr, half8 *Av = nullptr,
                                           Slice slice = Slice())
{
    constexpr bool KLO = LO != kLoNone;
    // KLO: the keys carry the softmax constant (see prefill_dequantize) and the accumulators start from init[qt] = minus
    // the query's reference maximum, four times: the products come out in the exponent's units, relative to the
    // reference, and the common case of the softmax has neither a multiplication nor a subtraction left to do.
    // Otherwise (fp16 rows: window chunks, 16-bit keys) they start from zero and the scores are raw.
    // Operands come from LDS one batch (two rows x 8 channels per lane = 8 registers) at a time, two batches ahead of the
    // products that use them; a compiler barrier per batch keeps the order (left alone, the compiler either fetches all
    // 64 registers of a unit up front or waits for every batch right after asking for it).  With Xv: the value
    // operands of the output product that follows (unit Xv) are asked for during the last batches, so that they are
    // there when the softmax is done.
    // slice(bt): vector work of another unit (a share of its softmax) that is to be issued between the products of batch
    // bt and those of the next; with one, nothing is moved across the end of a batch (left alone, the compiler puts all
    // of it behind the last products, where the matrix cores then idle).
    constexpr int kBatches = score_batches<LO>();
    auto fetch = [&](int bt, half8 &A0, half8 &A1) {
        const int step = bt & 3;
        if (LO == kLoCompact && bt >= 4) {
            const _Float16 *lo = &X.Klo[0][0];
            A0 = *reinterpret_cast<const half8 *>(lo + n * kLoStride + 8 * rq);
            A1 = *reinterpret_cast<const half8 *>(lo + (16 + n) * kLoStride + 8 * rq);
        } else if (KLO && bt >= 4) {
            A0 = *reinterpret_cast<const half8 *>(&X.Klo[n][32 * step + 8 * rq]);
            A1 = *reinterpret_cast<const half8 *>(&X.Klo[16 + n][32 * step + 8 * rq]);
        } else {
            A0 = *reinterpret_cast<const half8 *>(&X.K[n][32 * step + 8 * rq]);
            A1 = *reinterpret_cast<const half8 *>(&X.K[16 + n][32 * step + 8 * rq]);
        }
    };
    half8 A0[kBatches], A1[kBatches];
    constexpr int kAhead = 2;                                   // batches in flight (2..4 measured alike)
#pragma unroll
    for (int bt = 0; bt < kAhead && bt < kBatches; bt++) fetch(bt, A0[bt], A1[bt]);
    constexpr int kVFirst = kBatches - 2;                       // the value operands ride with the last two batches
#pragma unroll
    for (int bt = 0; bt < kBatches; bt++) {
        if (bt + kAhead < kBatches) fetch(bt + kAhead, A0[bt + kAhead], A1[bt + kAhead]);
        if (Xv && bt >= kVFirst && bt < kVFirst + 2) {
#pragma unroll
            for (int k = 0; k < 4; k++) Av[4 * (bt - kVFirst) + k] = value_operand(*Xv, 4 * (bt - kVFirst) + k, n, rq);
        }
        asm volatile("" ::: "memory");
        const int step = bt & 3;
#pragma unroll
        for (int qt = 0; qt < kQT; qt++) {
            const float4v start = KLO ? init[qt] : float4v{0.0f, 0.0f, 0.0f, 0.0f};
            const half8 B = LO == kLoCompact && bt >= 4 ? Qlo[qt] : Qf[qt][step];
            S[0][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A0[bt], B, bt == 0 ? start : S[0][qt], 0, 0, 0);
            S[1][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A1[bt], B, bt == 0 ? start : S[1][qt], 0, 0, 0);
        }
        if constexpr (!std::is_same<Slice, NoSlice>::value) {
            slice(bt);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// acc + the sum of the eight weights as they enter the output product (rounded to fp16), in fp32: four two-element dot
// products.  The denominator then matches the numerators exactly.
__device__ __forceinline__ float add_weights(float acc, half8 P)
{
    typedef _Float16 half2 __attribute__((ext_vector_type(2)));
    const half2 ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
    for (int k = 0; k < 4; k++) acc = __builtin_amdgcn_fdot2(half2{P[2 * k], P[2 * k + 1]}, ones, acc, false);
    return acc;
}

// The reference m of a query (in the exponent's units: score * log2(e) / sqrt(D)) only has to keep the weights in range,
// it need not be the exact maximum: as long as no score exceeds it by more than kCalm, it stays (no rescaling, weights
// <= 2^kCalm: fp16 holds them, the accumulators are fp32).
constexpr float kCalm = 8.0f;

// Online softmax in base 2 of the unit's scores, exact form: weights P (fp16, already in the operand order of the output
// product), reference m, partial sums lsum, and the factors alpha by which the accumulators shrink.  Returns whether
// some reference moved (in any lane).
// PRE: the scores are in the exponent's units and relative to base[qt] (score_unit with KLO); otherwise raw: the
// exponent is score * c + base[qt].
// MASK: the unit reaches beyond some query's position.
template <bool MASK, bool PRE>
__device__ __forceinline__ bool softmax_unit(const float4v (&S)[2][kQT], float c, int u, const int (&qpos)[kQT], const float (&base)[kQT],
                                             float (&m)[kQT], float (&lsum)[kQT], half8 (&P)[kQT], float (&alpha)[kQT], int rq)
{
    bool moved = false;
#pragma unroll
    for (int qt = 0; qt < kQT; qt++) {
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; e++) x[e] = S[e >> 2][qt][e & 3];
        if constexpr (MASK) {
#pragma unroll
            for (int e = 0; e < 8; e++)
                if (32 * u + 16 * (e >> 2) + 4 * rq + (e & 3) > qpos[qt]) x[e] = -INFINITY;
        }
        float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
        mx = fmaxf(mx, xor_lanes(mx, 16));
        mx = fmaxf(mx, xor_lanes(mx, 32));
        // unit 0 holds token 0, which every query sees: the reference is finite from the start
        const float top = PRE ? mx + base[qt] : fmaf(mx, c, base[qt]);
        const float mn = top > m[qt] + kCalm ? top : m[qt];              // m = -inf at the start: moves
        moved |= mn != m[qt];
        alpha[qt] = __builtin_amdgcn_exp2f(m[qt] - mn);
        m[qt] = mn;
        const float shift = base[qt] - mn;
#pragma unroll
        for (int e = 0; e < 8; e++) x[e] = __builtin_amdgcn_exp2f(PRE ? x[e] + shift : fmaf(x[e], c, shift));
        P[qt] = half8{(_Float16)x[0], (_Float16)x[1], (_Float16)x[2], (_Float16)x[3],
                      (_Float16)x[4], (_Float16)x[5], (_Float16)x[6], (_Float16)x[7]};
        lsum[qt] = add_weights(lsum[qt] * alpha[qt], P[qt]);
    }
    return __any(moved);
}

// true if some score of the unit (no mask) exceeds its query's reference by more than kCalm, in any lane of the wave.
// PRE: the scores are relative to the reference already; otherwise raw (compared against (m + kCalm) / c).
template <bool PRE>
__device__ __forceinline__ bool unit_exceeds(const float4v (&S)[2][kQT], float inv_c, const float (&m)[kQT])
{
    bool over = false;
#pragma unroll
    for (int qt = 0; qt < kQT; qt++) {
        const float4v a = S[0][qt], b = S[1][qt];
        float mx = fmaxf(fmaxf(a[0], a[1]), a[2]);          // chains of three-operand maxima
        mx = fmaxf(fmaxf(mx, a[3]), b[0]);
        mx = fmaxf(fmaxf(mx, b[1]), b[2]);
        mx = fmaxf(mx, b[3]);
        over |= PRE ? mx > kCalm : mx > (m[qt] + kCalm) * inv_c;
    }
    return __any(over);
}

// Softmax weights of a unit against the unchanged reference (no mask), dealt out in kBatches shares so that a share
// can be issued between two batches of another unit's score products.  PRE: the scores are the exponents themselves.
template <bool PRE, int SHARES>
struct CalmSoftmax {
    const float4v (&S)[2][kQT];
    float c;
    const float (&m)[kQT];
    float (&lsum)[kQT];
    half8 (&P)[kQT];
    static constexpr int kShares = SHARES;                      // = the batches of the score products it rides with
    __device__ __forceinline__ void operator()(int share) const
    {
        typedef _Float16 half2 __attribute__((ext_vector_type(2)));
        const half2 ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
        for (int pair = 8 * share / kShares; pair < 8 * (share + 1) / kShares; pair++) {
            const int qt = pair >> 2, e = 2 * (pair & 3);                                       // elements e, e + 1 of query tile qt
            const float s0 = S[e >> 2][qt][e & 3], s1 = S[e >> 2][qt][(e & 3) + 1];
            const float x0 = __builtin_amdgcn_exp2f(PRE ? s0 : fmaf(s0, c, -m[qt]));
            const float x1 = __builtin_amdgcn_exp2f(PRE ? s1 : fmaf(s1, c, -m[qt]));
            const half2 h = {(_Float16)x0, (_Float16)x1};
            P[qt][e] = h[0];
            P[qt][e + 1] = h[1];
            // the denominator is summed from the rounded weights, as they enter the output product
            lsum[qt] = __builtin_amdgcn_fdot2(h, ones, lsum[qt], false);
        }
    }
};

// O^T += V^T P^T: rows = channels 16 ct + 4 rq + r; both operands list the tokens as
// {4 rq .. 4 rq + 3, 16 + 4 rq .. 16 + 4 rq + 3}.
__device__ __forceinline__ void output_add(const half8 (&Av)[8], const half8 (&P)[kQT], float4v (&O)[8][kQT])
{
#pragma unroll
    for (int ct = 0; ct < 8; ct++)
#pragma unroll
        for (int qt = 0; qt < kQT; qt++) O[ct][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(Av[ct], P[qt], O[ct][qt], 0, 0, 0);
}

// O^T *= alpha per query, before the unit's product is added (on the exact path only, which is the rare one).
__device__ __forceinline__ void output_rescale(const float (&alpha)[kQT], float4v (&O)[8][kQT])
{
#pragma unroll
    for (int qt = 0; qt < kQT; qt++)
#pragma unroll
        for (int ct = 0; ct < 8; ct++) O[ct][qt] *= alpha[qt];
}

// ---- pass 0 (per-channel quantized keys only): which channels of each cache keep the low parts of their keys.
// A key rounded once to fp16 is off by up to 2^-11 of itself, and the logit by the sum over the channels of that times
// the query's entry.  Per channel d this kernel estimates the centre of the dequantized keys (the mean of the blocks'
// midpoints, rounded to fp16) and w_d = (mean square of the keys about that centre) x (mean square of the queries):
// the keys' from the block metadata alone (a block's values of a channel lie in [z, z + s (2^bits - 1)],
// taken as spread evenly), the queries' from up to 64 positions of every query head of the group.  The 32 channels of
// largest w_d keep their low parts; if the w_d of all others add up to less than kSelectBudget, i.e. one fp16 rounding
// of those channels moves a logit by less than 2^-11 / sqrt(3) * log2(e) / sqrt(D) * sqrt(kSelectBudget) = 6e-4 (root
// mean square, in the exponent's units: below the 2^-11 by which the fp16 softmax weights are rounded anyway), the
// cache takes the compact form; otherwise every channel keeps its low part.  Keys whose large channels are few
// (the case the per-channel grouping is made for, Section 3.2) qualify, and so do keys with a large offset on every
// channel (the offsets are centred away); keys that are large and widely spread on many channels do not.
constexpr float kSelectBudget = 300.0f;
constexpr int kSelectParts = 8;

template <bool NARROW>
__global__ __launch_bounds__(kD * kSelectParts) void prefill_select(PrefillArgs a)
{
    const int d = threadIdx.x & (kD - 1), part = threadIdx.x >> 7, local = blockIdx.x, bh = a.bh0 + local;
    __shared__ float k1[kSelectParts][kD], k2[kSelectParts][kD], q2[kSelectParts][kD], w[kD], rest[kD];
    const float top = (float)((1 << a.lv.kbits) - 1);
    float sk = 0.0f, sm = 0.0f;
    for (int u0 = part; u0 < a.n_blocks; u0 += 4 * kSelectParts) {
        float sc[4], zp[4];
#pragma unroll
        for (int k = 0; k < 4; k++) {                            // four blocks in flight
            const int u = u0 + kSelectParts * k < a.n_blocks ? u0 + kSelectParts * k : u0;
            const float *meta = a.lv.kmeta + ((size_t)bh * a.NB + u) * meta_words(NARROW);
            sc[k] = NARROW ? half_bits(meta_scales16(meta)[d]) : meta[d];
            zp[k] = half_bits(meta_zeros(meta, NARROW)[d]);
        }
#pragma unroll
        for (int k = 0; k < 4; k++) {
            if (u0 + kSelectParts * k < a.n_blocks) {
                const float lo = zp[k], hi = fmaf(sc[k], top, lo);
                sk += (lo * lo + lo * hi + hi * hi) * (1.0f / 3.0f);        // mean of x^2 over [lo, hi]
                sm += 0.5f * (lo + hi);
            }
        }
    }
    const int gq = a.Hq / a.Hkv, stride = (a.n_q + 63) / 64;
    const int head0 = (bh / a.Hkv) * a.Hq + (bh % a.Hkv) * gq;
    const int per_head = (a.n_q + stride - 1) / stride, samples = gq * per_head;
    float sq = 0.0f;
    for (int i0 = part; i0 < samples; i0 += 8 * kSelectParts) {
        uint16_t x[8];
#pragma unroll
        for (int k = 0; k < 8; k++) {                            // eight samples in flight
            const int i = i0 + kSelectParts * k < samples ? i0 + kSelectParts * k : i0;
            x[k] = a.q[((size_t)(head0 + i / per_head) * a.n_q + (size_t)(i % per_head) * stride) * kD + d];
        }
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const float v = i0 + kSelectParts * k < samples ? half_bits(x[k]) : 0.0f;
            sq = fmaf(v, v, sq);
        }
    }
    k1[part][d] = sm;
    k2[part][d] = sk;
    q2[part][d] = sq;
    __syncthreads();
    Select *sel = reinterpret_cast<Select *>(a.select) + local;
    if (part == 0) {
        float tm = 0.0f, tk = 0.0f, tq = 0.0f;
#pragma unroll
        for (int k = 0; k < kSelectParts; k++) { tm += k1[k][d]; tk += k2[k][d]; tq += q2[k][d]; }
        // the channel's centre: the mean of its blocks' midpoints, as an fp16 number (the zero-points are fp16 numbers, so
        // zero-point minus centre is exact in fp32).  What counts from here on is the keys' spread about it.
        const float centre = (float)(_Float16)(tm / (float)a.n_blocks);
        const float centre_ok = fabsf(centre) < 65504.0f ? centre : 0.0f;
        sel->centre[d] = centre_ok;
        const float spread = fmaxf(tk / (float)a.n_blocks - centre_ok * (2.0f * tm / (float)a.n_blocks - centre_ok), 0.0f);
        w[d] = spread * (tq / (float)samples);
    }
    __syncthreads();
    if (part == 0) {
        const float mine = w[d];
        int rank = 0;
        for (int o = 0; o < kD; o++) rank += (w[o] > mine || (w[o] == mine && o < d)) ? 1 : 0;
        sel->pos[d] = rank < 32 ? (uint8_t)rank : (uint8_t)255;
        if (rank < 32) sel->chan[rank] = (uint8_t)d;
        rest[d] = rank < 32 && mine == mine ? 0.0f : mine;       // (not a number: stays one, and the sum below with it)
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float r = 0.0f;
        for (int o = 0; o < kD; o++) r += rest[o];
        sel->compact = r < kSelectBudget ? 1u : 0u;              // (a sum that is not a number compares false: all channels)
    }
}

// ---- pass 1: every packed unit of the (batch, kv head) caches [bh0, bh0 + n_bh) is dequantized once into the scratch
// area, in the very layout the attention kernel keeps a unit in LDS (struct Tiles), so that pass 2 fetches plain copies.
// KQ / VQ: the layer's keys / values are quantized (else fp16 rows in the code area).
template <bool KQ, bool VQ>
__global__ __launch_bounds__(64 * kStagers) void prefill_dequantize(PrefillArgs a)
{
    const int tid = threadIdx.x, u = blockIdx.x, local = blockIdx.y;
    const int T = 32 * a.n_blocks + a.n_res;
    __shared__ __attribute__((aligned(16))) MetaSlab M[kStagers];
    Stage st;
    load_packed<KQ, VQ>(a, a.bh0 + local, u, T, tid, st);
    const Select *rec = KQ && a.select ? reinterpret_cast<const Select *>(a.select) + local : nullptr;
    Tiles &dst = *reinterpret_cast<Tiles *>(a.scratch + ((size_t)local * a.n_blocks + u) * sizeof(Tiles));
    store_packed<KQ, VQ>(a, tid, st, dst, M[tid >> 6], rec);
}

// A unit goes from the scratch area into an LDS buffer without passing through registers: a wave issues
// global-to-LDS loads of 1 KiB each (64 lanes x 16 bytes, which land at consecutive LDS addresses from the base
// that M0 holds).  The three tiles of a unit are 9 KiB each, so a piece never straddles two of them.
constexpr int kTileKiB = 9;
static_assert(sizeof(_Float16) * 32 * kKStride == kTileKiB * 1024 && sizeof(_Float16) * kD * kVStride == kTileKiB * 1024 &&
              sizeof(Tiles) == 3 * kTileKiB * 1024, "tiles of a unit are whole KiB");

__device__ __forceinline__ void fetch_piece(const uint8_t *unit, uint32_t offset_of_lane, uint32_t lds_base)
{
    // The compiler does not see this load: the waits for it are written out below (wait_fetches).  Loads it does not
    // know of can only make its own waits longer, never too short.  M0 is declared as clobbered, so a use of its own the compiler
    // might make of M0 (it sets M0 right before an instruction that reads it) stays correct.
    // Address = the unit's (wave-uniform, scalar registers) + a 32-bit offset per lane that is the same for every unit.
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(offset_of_lane), "s"(unit) : "memory", "m0");
}

// Wave `wave` fetches the pieces wave, wave + 8, ... of a unit.  Of the keys' low parts: none, the whole tile, or the
// first kLoPieces KiB of it (the compact tile).
template <int LO>
__device__ __forceinline__ void fetch_unit(const uint8_t *unit, Tiles &L, int wave, int lane)
{
    constexpr int lo_pieces = LO == kLoAll ? kTileKiB : LO == kLoCompact ? kLoPieces : 0;
    constexpr int pieces = 2 * kTileKiB + lo_pieces;
    const uint32_t lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)reinterpret_cast<uint8_t *>(&L);
#pragma unroll
    for (int i = 0; i < (pieces + kWaves - 1) / kWaves; i++) {
        const int p = wave + kWaves * i;                          // the same for all lanes of the wave
        if (p < pieces) {
            const int off = 1024 * (p < kTileKiB + lo_pieces ? p : p - lo_pieces + kTileKiB);     // K^, low parts, then V^
            fetch_piece(unit, (uint32_t)(off + 16 * lane), lds + off);
        }
    }
}

// Returns once all fetches of this wave have landed in LDS.
__device__ __forceinline__ void wait_fetches() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---- pass 2: the attention itself.  One work-group per 256 consecutive queries of one query head; every wave attends
// 32 queries and fetches its share of each unit from the scratch area into LDS.  KLO: the keys are quantized (they come
// as two fp16 numbers).
//
// Five LDS buffers and two units per trip: while units u and u + 1 are being used, unit u + 2 is already there and units
// u + 3 and u + 4 are on their way; one barrier per trip.  With the next unit present, a wave issues the score products
// of unit u + 1 in the same stretch of code as the softmax of unit u (matrix and vector instructions that do not depend
// on each other), instead of waiting for each product's result in turn.
constexpr int kBuffers = 5;

// LO: how the low parts of the keys come (score_unit); rec: the cache's selection record or null (never null with
// kLoCompact).
template <int LO>
__device__ __forceinline__ void attend(const PrefillArgs &a, const Select *rec, int local, int jq, int rank)
{
    constexpr bool KLO = LO != kLoNone;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, rq = lane >> 4;
    const int tiles = (a.n_q + kQB - 1) / kQB;
    const int gq = a.Hq / a.Hkv;
    const int bh = a.bh0 + local;
    const int tile = tiles - 1 - rank;                           // the longest rows start first
    const int head = (bh / a.Hkv) * a.Hq + (bh % a.Hkv) * gq + jq;   // b * Hq + query head
    const int T = 32 * a.n_blocks + a.n_res;
    const int p0 = T - a.n_q;                                    // absolute position of query 0
    const int i0 = tile * kQB;
    const int ilast = (i0 + kQB < a.n_q ? i0 + kQB : a.n_q) - 1;
    const int units = (p0 + ilast) / 32 + 1;                     // units the work-group walks through
    const int iw = i0 + kQW * wave;                              // first query of this wave
    const int wlast = iw < a.n_q ? (p0 + (iw + kQW - 1 < a.n_q ? iw + kQW - 1 : a.n_q - 1)) / 32 : -1;
    const int wmin = p0 + iw;                                    // position of the wave's first query
    const int open_units = iw < a.n_q ? (wmin + 1) / 32 : 0;     // units [0, open_units) lie before it: no mask needed
    const float c = a.scale_log2e;
    const float inv_c = 1.0f / c;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    Tiles *L = reinterpret_cast<Tiles *>(lds_raw);

    // queries of this lane: iq[qt] = iw + 16 qt + n; past the end the last query is repeated and never stored
    int qpos[kQT];
    half8 Qf[kQT][4], Qlo[kQT];
#pragma unroll
    for (int qt = 0; qt < kQT; qt++) {
        const int i = iw + 16 * qt + n, ic = i < a.n_q ? i : a.n_q - 1;
        qpos[qt] = p0 + ic;
        const uint16_t *row = a.q + ((size_t)head * a.n_q + ic) * kD;
#pragma unroll
        for (int step = 0; step < 4; step++) Qf[qt][step] = __builtin_nontemporal_load(reinterpret_cast<const half8 *>(row + 32 * step + 8 * rq));
        if constexpr (LO == kLoCompact) {
            // the query's values at the channels of slots 8 rq .. 8 rq + 7: the operand that meets the compact tile
            const u32x2 cw = *reinterpret_cast<const u32x2 *>(&rec->chan[8 * rq]);
#pragma unroll
            for (int e = 0; e < 8; e++)
                Qlo[qt][e] = __builtin_bit_cast(_Float16, row[((e < 4 ? cw[0] : cw[1]) >> (8 * (e & 3))) & 127u]);
        } else {
            Qlo[qt] = half8{};
        }
    }

    // Packed keys come with their channel's centre taken off (prefill_dequantize), which lowers every packed score of a
    // query by q . centre; the scores of the window's fp16 rows are lowered by the same amount here, so that the softmax
    // sees all of a query's scores moved alike.  woff = minus that amount in the exponent's units.
    float woff[kQT];
#pragma unroll
    for (int qt = 0; qt < kQT; qt++) woff[qt] = 0.0f;
    if constexpr (KLO) {
        if (rec) {
#pragma unroll
            for (int qt = 0; qt < kQT; qt++) {
                float dot = 0.0f;
#pragma unroll
                for (int step = 0; step < 4; step++) {
                    const float4 c0 = *reinterpret_cast<const float4 *>(&rec->centre[32 * step + 8 * rq]);
                    const float4 c1 = *reinterpret_cast<const float4 *>(&rec->centre[32 * step + 8 * rq + 4]);
                    const float cen[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
                    for (int e = 0; e < 8; e++) dot = fmaf((float)Qf[qt][step][e], cen[e], dot);
                }
                dot += xor_lanes(dot, 16);
                dot += xor_lanes(dot, 32);
                woff[qt] = -c * dot;
            }
        }
    }

    float4v O[8][kQT];
    float m[kQT], lsum[kQT];
#pragma unroll
    for (int qt = 0; qt < kQT; qt++) {
        m[qt] = -INFINITY;
        lsum[qt] = 0.0f;
#pragma unroll
        for (int ct = 0; ct < 8; ct++) O[ct][qt] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
    }

    // ---- packed units [0, nb).  Unit u lives in buffer u % 5.  Per trip: the wave issues its fetches of units u + 3 and
    // u + 4 (into the buffers of units u - 2 and u - 1, which everybody left at the last barrier), uses units u and u + 1
    // (taking the scores of the following unit ahead each time), then waits until its fetches have landed, and the
    // barrier makes everybody's visible.  Past the end the last unit is fetched again, into a buffer nobody reads.
    const int nb = a.n_blocks < units ? a.n_blocks : units;
    if (nb > 0) {
        const uint8_t *mine = a.scratch + (size_t)local * a.n_blocks * sizeof(Tiles);
        const int last = nb - 1;
        auto unit_at = [&](int u) { return mine + (size_t)(u < last ? u : last) * sizeof(Tiles); };
        fetch_unit<LO>(unit_at(0), L[0], wave, lane);
        fetch_unit<LO>(unit_at(1), L[1], wave, lane);
        fetch_unit<LO>(unit_at(2), L[2], wave, lane);
        // The queries are first used under a condition; without this the compiler would keep their loads on its list
        // of pending ones inside the loop and wait there for everything in flight, the fetches just issued included.
#pragma unroll
        for (int qt = 0; qt < kQT; qt++)
#pragma unroll
            for (int step = 0; step < 4; step++) asm volatile("" ::"v"(Qf[qt][step]));
        if constexpr (LO == kLoCompact) {
#pragma unroll
            for (int qt = 0; qt < kQT; qt++) asm volatile("" ::"v"(Qlo[qt]));
        }
        wait_fetches();                                         // units 0, 1 and 2 are there
        __syncthreads();
        float4v S[2][kQT], Sn[2][kQT];
        // base[qt]: what the scores waiting in S / Sn are relative to (KLO only: the reference as it stood when their
        // products were issued, zero while it is still -inf); init = minus that, as the products' starting value
        float base[kQT];
        float4v init[kQT];
        auto set_base = [&]() {
#pragma unroll
            for (int qt = 0; qt < kQT; qt++) {
                base[qt] = KLO && m[qt] > -INFINITY ? m[qt] : 0.0f;
                init[qt] = float4v{-base[qt], -base[qt], -base[qt], -base[qt]};
            }
        };
        set_base();
        if (0 <= wlast) score_unit<LO>(L[0], Qf, Qlo, S, n, rq, init);
        // one unit: its scores come in Sin, those of the next unit leave in Sout (the two arrays swap roles from unit to
        // unit).  Whether a unit may take the calm form is decided one unit ahead, right after its scores were issued:
        // the test then sits next to the output products of the unit before, which need nothing from it.
        bool calm = false;                                       // unit 0 never is: the references start at -inf
        auto step = [&](int u, const Tiles &X0, const Tiles &X1, const float4v (&Sin)[2][kQT], float4v (&Sout)[2][kQT]) {
            if (u <= wlast) {
                const bool ahead = u + 1 < nb && u + 1 <= wlast;
                half8 P[kQT];
                float alpha[kQT];
                const bool was_calm = calm;
                bool moved = false;                              // some reference moved after the next unit's scores were issued
                half8 Av[8];
                if (calm) {
                    // the common case, one stretch of straight-line code: score products of the next unit next to the
                    // weights of this one against the unchanged reference (calm implies that there is a next unit, and
                    // that this unit's scores are relative to the reference as it stands: base, init are up to date)
                    score_unit<LO>(X1, Qf, Qlo, Sout, n, rq, init, &X0, Av, CalmSoftmax<KLO, score_batches<LO>()>{Sin, c, m, lsum, P});
                } else {
                    float bin[kQT];
#pragma unroll
                    for (int qt = 0; qt < kQT; qt++) bin[qt] = base[qt];
                    if (ahead) {
                        set_base();
                        score_unit<LO>(X1, Qf, Qlo, Sout, n, rq, init, &X0, Av);
                    } else {
#pragma unroll
                        for (int ct = 0; ct < 8; ct++) Av[ct] = value_operand(X0, ct, n, rq);
                    }
                    if (u < open_units) moved = softmax_unit<false, KLO>(Sin, c, u, qpos, bin, m, lsum, P, alpha, rq);
                    else moved = softmax_unit<true, KLO>(Sin, c, u, qpos, bin, m, lsum, P, alpha, rq);
                }
                // The accumulators are touched under a condition of their own, not inside the two-sided one above: there
                // the compiler's merge block sits in front of the calm side, and the calm side then copied all 64
                // accumulator registers, every unit, to meet the rescaled ones.
                if (!was_calm) output_rescale(alpha, O);
                // one place adds to the accumulators on every path: they stay in the same registers (with a product
                // on each path the compiler copied all 64 of them after every unit)
                output_add(Av, P, O);
                // the next unit is calm if it needs no mask, has a unit after it to look ahead to, its scores are
                // relative to the reference as it stands now, and none of them exceeds it by more than kCalm
                calm = ahead && u + 2 < nb && u + 2 <= wlast && u + 1 < open_units && !(KLO && moved) && !unit_exceeds<KLO>(Sout, inv_c, m);
            }
        };
        auto after = [](int x) { return x + 1 < kBuffers ? x + 1 : 0; };
        int b0 = 0;                                              // buffer of unit u
        for (int u = 0; u < nb; u += 2) {
            const int b1 = after(b0), b2 = after(b1), b3 = after(b2), b4 = after(b3);
            fetch_unit<LO>(unit_at(u + 3), L[b3], wave, lane);  // buffers of units u - 2 and u - 1: all are done with them
            fetch_unit<LO>(unit_at(u + 4), L[b4], wave, lane);
            step(u, L[b0], L[b1], S, Sn);
            if (u + 1 < nb) step(u + 1, L[b1], L[b2], Sn, S);
            wait_fetches();                                     // units u + 3 and u + 4 are there
            __syncthreads();
            b0 = b2;
        }
    }
    // ---- chunks of the fp16 window, staged by the first four waves straight from the ring
    for (int u = nb; u < units; u++) {
        if (wave < kStagers) stage_window(a, bh, u, T, tid, L[0]);
        __syncthreads();
        if (u <= wlast) {
            float4v S[2][kQT];
            half8 P[kQT];
            float alpha[kQT];
            const float4v none[kQT] = {};
            score_unit<kLoNone>(L[0], Qf, Qlo, S, n, rq, none);                 // fp16 rows: raw scores
            softmax_unit<true, false>(S, c, u, qpos, woff, m, lsum, P, alpha, rq);
            output_rescale(alpha, O);
            half8 Av[8];
#pragma unroll
            for (int ct = 0; ct < 8; ct++) Av[ct] = value_operand(L[0], ct, n, rq);
            output_add(Av, P, O);
        }
        __syncthreads();
    }

#pragma unroll
    for (int qt = 0; qt < kQT; qt++) {
        float l = lsum[qt];
        l += xor_lanes(l, 16);
        l += xor_lanes(l, 32);
        const int i = iw + 16 * qt + n;
        if (i < a.n_q) {
            const float inv = 1.0f / l;
            uint16_t *row = a.out + ((size_t)head * a.n_q + i) * kD;
#pragma unroll
            for (int ct = 0; ct < 8; ct++)
                __builtin_nontemporal_store(u32x2{pack2(O[ct][qt][0] * inv, O[ct][qt][1] * inv), pack2(O[ct][qt][2] * inv, O[ct][qt][3] * inv)},
                                            reinterpret_cast<u32x2 *>(row + 16 * ct + 4 * rq));
        }
    }
}

// KQ: the layer's keys are quantized.  Each cache of such a layer is attended in the form its selection record names
// (without records: low parts of all channels).
template <bool KQ>
__global__ __launch_bounds__(64 * kWaves, 1) void prefill_attention(PrefillArgs a)
{
    const int tiles = (a.n_q + kQB - 1) / kQB;
    const int gq = a.Hq / a.Hkv;
    // Work-groups go to the 8 XCDs in turn by their index, and each XCD has an L2 of its own: all query heads and
    // query tiles that read one (batch, kv head) cache are given to one XCD (when the count divides), so that its
    // units are fetched from memory once and then served by that L2.
    int local, jq, rank;                                         // cache within this launch, query head within its group, order
    if (a.n_bh % 8 == 0) {
        const int xcd = blockIdx.x & 7, k = blockIdx.x >> 3, per = gq * tiles;
        local = 8 * (k / per) + xcd;
        jq = (k % per) % gq;
        rank = (k % per) / gq;
    } else {
        local = blockIdx.x / (gq * tiles);
        jq = (blockIdx.x / tiles) % gq;
        rank = blockIdx.x % tiles;
    }
    if constexpr (KQ) {
        const Select *rec = a.select ? reinterpret_cast<const Select *>(a.select) + local : nullptr;
        if (rec && __builtin_amdgcn_readfirstlane((int)rec->compact) != 0) attend<kLoCompact>(a, rec, local, jq, rank);
        else attend<kLoAll>(a, rec, local, jq, rank);
    } else {
        attend<kLoNone>(a, nullptr, local, jq, rank);
    }
}

}  // namespace


size_t prefill_unit_bytes() { return sizeof(Tiles); }
size_t prefill_select_bytes() { return sizeof(Select); }

// Pass 0 for the caches [bh0, bh0 + n_bh) (a.select = their first record); only for layers whose keys are quantized
// per channel and hold packed blocks.  ev_begin (may be null) receives the kernel's start.
hipError_t launch_prefill_select(const PrefillArgs &a, hipStream_t s, hipEvent_t ev_begin)
{
    if (!a.select || a.lv.kbits >= 16 || a.lv.kpt || a.n_blocks < 1 || a.n_bh < 1) return hipErrorInvalidValue;
    const dim3 grid((unsigned)a.n_bh), block(kD * kSelectParts);
    auto launch = [&](auto kernel) {
        if (ev_begin) hipExtLaunchKernelGGL(kernel, grid, block, 0, s, ev_begin, nullptr, 0, a);
        else hipLaunchKernelGGL(kernel, grid, block, 0, s, a);
    };
    if (a.lv.narrow) launch(prefill_select<true>);
    else launch(prefill_select<false>);
    return hipGetLastError();
}

hipError_t launch_prefill_attention(const PrefillArgs &a, hipStream_t s, hipEvent_t ev_begin, hipEvent_t ev_end)
{
    const long long tiles = (a.n_q + kQB - 1) / kQB;
    const long long groups = tiles * a.n_bh * (a.Hq / a.Hkv);
    if (groups < 1 || groups > 0x7fffffffLL || a.n_bh < 1 || a.n_bh > 65535) return hipErrorInvalidConfiguration;
    const bool kq = a.lv.kbits < 16, vq = a.lv.vbits < 16;
    // selection records only exist where launch_prefill_select could write them
    if (a.select && !(kq && !a.lv.kpt && a.n_blocks > 0)) return hipErrorInvalidValue;
    hipEvent_t begin = ev_begin;                                 // stamped by the start of the first kernel launched
    if (a.n_blocks > 0) {
        // pass 1
        const dim3 grid((unsigned)a.n_blocks, (unsigned)a.n_bh), block(64 * kStagers);
        auto launch = [&](auto kernel) {
            if (begin) hipExtLaunchKernelGGL(kernel, grid, block, 0, s, begin, nullptr, 0, a);
            else hipLaunchKernelGGL(kernel, grid, block, 0, s, a);
            begin = nullptr;
        };
        if (kq && vq) launch(prefill_dequantize<true, true>);
        else if (kq) launch(prefill_dequantize<true, false>);
        else if (vq) launch(prefill_dequantize<false, true>);
        else launch(prefill_dequantize<false, false>);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // pass 2 (kBuffers tile buffers: more LDS than a kernel may declare statically)
    const dim3 grid((unsigned)groups), block(64 * kWaves);
    const size_t lds = kBuffers * sizeof(Tiles);
    auto attend_launch = [&](auto kernel) -> hipError_t {
        // the larger dynamic LDS size is asked for at every launch of either kernel, on whichever device is current:
        // a host-side setting, negligible next to a launch of milliseconds, and no process-wide state to keep
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        if (begin || ev_end) hipExtLaunchKernelGGL(kernel, grid, block, lds, s, begin, ev_end, 0, a);
        else hipLaunchKernelGGL(kernel, grid, block, lds, s, a);
        return hipGetLastError();
    };
    return kq ? attend_launch(prefill_attention<true>) : attend_launch(prefill_attention<false>);
}

}  // namespace kvq
