// Quantize-and-pack kernels: Section 3.2, Eq. 2 of the paper applied KIVI-style
// (keys per channel over the 32 tokens of a block, values per token over each 32
// channels), the fp16 window copy, and the canonical export used by tests.
//
// The encode arithmetic is fixed so that every implementation produces the same
// bits: fp16 inputs widened to fp32, z = min, s = (max - min) / (2^B - 1) with one
// IEEE subtraction and one IEEE division, code = clamp(rne((x - z) / s), 0, 2^B - 1)
// with one IEEE subtraction, one IEEE division and round-half-to-even; s == 0 gives
// code 0.  This file is compiled without floating-point contraction.
#include "kvq_internal.h"

namespace kvq {
namespace {

__device__ __forceinline__ float half_bits_to_float(uint32_t h)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}

// bit pattern of a float that is known to be an fp16 number (a minimum of fp16 inputs): the narrowing is exact
__device__ __forceinline__ uint16_t float_to_half_bits_exact(float x)
{
    return __builtin_bit_cast(uint16_t, (_Float16)x);
}

// fp16 row of the token at absolute position pos: the window ring for tokens that were
// already held, the caller's tensor for tokens of this append.
__device__ __forceinline__ const uint16_t *token_row(const uint16_t *in, const uint16_t *ring, int bh, int pos,
                                                     int t_old, int n_in, int RC)
{
    return pos < t_old ? ring + ((size_t)bh * RC + pos % RC) * kD
                       : in + ((size_t)bh * n_in + (pos - t_old)) * kD;
}

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// element-wise minimum / maximum of two fp16 pairs (exact; the statistics need no widening).  Written as
// single instructions: the generic vector builtins add a quieting pass over every loaded operand.
__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b)
{
    uint32_t d;
    asm("v_pk_min_f16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b)
{
    uint32_t d;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}

// Eq. 2 takes min(X) and max(X) as numbers, and the number zero has two encodings.  A zero extreme is stored as +0
// whichever zeros the group holds and in whichever order the reduction met them, so that z and s have one bit pattern.
__device__ __forceinline__ uint32_t plus_zero_pair(uint32_t w)
{
    if ((w & 0x00007fffu) == 0) w &= 0xffff0000u;
    if ((w & 0x7fff0000u) == 0) w &= 0x0000ffffu;
    return w;
}
__device__ __forceinline__ float plus_zero(float x) { return x == 0.0f ? 0.0f : x; }

// Eq. 2 for one element, the defining sequence: (one IEEE subtraction, done by the caller,) one IEEE
// division, round half to even, clamp.  Returns the code as a float.
template <int BITS>
__device__ __forceinline__ float round_exact(float d, float s)
{
    const float r = rintf(s != 0.0f ? __fdiv_rn(d, s) : 0.0f);
    return fminf(fmaxf(r, 0.0f), (float)((1 << BITS) - 1));
}

// Eight elements at once, codes returned as floats.  d * (1 / s) with the hardware reciprocal (1 ulp) differs
// from the correctly rounded quotient by less than 2^-22 of its value, so both round to the same integer
// unless the product lies that close to a tie; the test below uses twice that distance.  If it fires for any
// lane of the wave (rare for real data, always for exact ties) the caller redoes the eight elements with the
// defining division (redo8; only then are the scales themselves fetched).  d >= 0 and rs >= 0 (rs is 0 where s
// is 0, giving code 0), so the fast result needs no clamp from below, and none from above either while s is the
// fp32 scale: d / s <= (2^B - 1)(1 + 2^-23).  CLAMP is for the narrow-metadata variant, whose rounded scale can
// be too small.  Returns true if the redo is needed; d = x - z is handed back for it.
//
// x and z come as fp16 pairs.  d = fma(x, one, -z) with both widened exactly is the one IEEE subtraction of the
// definition; `one` is 1.0 in a register the compiler cannot see through, so that the widenings and the
// subtraction stay one mixed-precision instruction instead of three.
// The distance of t = d * rs from the nearest tie is 1/2 - |t - rint(t)| (both differences are exact).
template <int BITS, bool CLAMP>
__device__ __forceinline__ bool encode8(const uint32_t (&xw)[4], const uint32_t (&zw)[4], const float (&r8)[8], float one,
                                        float (&d)[8], float (&c8)[8])
{
    float u[8];
#pragma unroll
    for (int e = 0; e < 8; e++) {
        const half2v xh = __builtin_bit_cast(half2v, xw[e >> 1]), zh = __builtin_bit_cast(half2v, zw[e >> 1]);
        d[e] = __builtin_fmaf((float)xh[e & 1], one, -(float)zh[e & 1]);
        const float t = d[e] * r8[e];
        const float c = rintf(t);
        c8[e] = CLAMP ? fminf(c, (float)((1 << BITS) - 1)) : c;
        const float res = fabsf(t - c);
        // few levels: one margin for all, 2^-21 times an upper bound 2^B of the quotient; else 2^-21 t
        if constexpr (!CLAMP && BITS <= 4) u[e] = res;
        else u[e] = __builtin_fmaf(t, 4.76837158203125e-07f, res);
    }
    const float worst = fmaxf(fmaxf(fmaxf(u[0], u[1]), fmaxf(u[2], u[3])), fmaxf(fmaxf(u[4], u[5]), fmaxf(u[6], u[7])));
    if constexpr (!CLAMP && BITS <= 4) return __any(worst >= 0.5f - (float)(1 << BITS) * 4.76837158203125e-07f);
    else return __any(worst >= 0.5f);
}

template <int BITS>
__device__ __forceinline__ void redo8(const float (&d)[8], const float (&s8)[8], float (&c8)[8])
{
#pragma unroll
    for (int e = 0; e < 8; e++) c8[e] = round_exact<BITS>(d[e], s8[e]);
}

// The lane's codes 8*m .. 8*m + 7 (as floats) into their dwords.  The fields of a dword are assembled in
// floating point while the partial words stay below 2^24 (exact), then converted once.
template <int BITS>
__device__ __forceinline__ void pack8(const float (&c)[8], int m, uint32_t *dw)
{
    if constexpr (BITS == 8) {
        // code e in byte e % 4 of dword 2*m + e / 4
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const float w = fmaf(c[4 * h + 2], 65536.0f, fmaf(c[4 * h + 1], 256.0f, c[4 * h]));
            dw[2 * m + h] = (uint32_t)w | ((uint32_t)c[4 * h + 3] << 24);
        }
    } else if constexpr (BITS == 4) {
        // nibble (e >> 1) + 4 * (e & 1) of dword m
        const float lo = fmaf(c[6], 4096.0f, fmaf(c[4], 256.0f, fmaf(c[2], 16.0f, c[0])));
        const float hi = fmaf(c[7], 4096.0f, fmaf(c[5], 256.0f, fmaf(c[3], 16.0f, c[1])));
        dw[m] = (uint32_t)lo | ((uint32_t)hi << 16);
    } else {
        // field 4 * (m & 1) + (e >> 1) + 8 * (e & 1) of dword m / 2
        const float lo = fmaf(c[6], 64.0f, fmaf(c[4], 16.0f, fmaf(c[2], 4.0f, c[0])));
        const float hi = fmaf(c[7], 64.0f, fmaf(c[5], 16.0f, fmaf(c[3], 4.0f, c[1])));
        const uint32_t w = (uint32_t)fmaf(hi, 65536.0f, lo);
        if (m & 1) dw[m >> 1] |= w << 8; else dw[m >> 1] = w;
    }
}

__device__ __forceinline__ float scale_of(float mn, float mx, int bits)
{
    return __fdiv_rn(mx - mn, (float)((1 << bits) - 1));
}

// the scale as it is stored and used: fp32, or rounded once to fp16 (round half to even) in the narrow variant
template <bool NARROW>
__device__ __forceinline__ float stored_scale(float s)
{
    if constexpr (NARROW) return (float)(_Float16)s;
    return s;
}
template <bool NARROW>
__device__ __forceinline__ void store_scale(float *meta, int idx, float s)
{
    if constexpr (NARROW) meta_scales16(meta)[idx] = __builtin_bit_cast(uint16_t, (_Float16)s);
    else meta[idx] = s;
}

// two neighbouring scales (even index first) as one store
template <bool NARROW>
__device__ __forceinline__ void store_scale_pair(float *meta, int idx, float s0, float s1)
{
    if constexpr (NARROW) {
        const uint32_t lo = __builtin_bit_cast(uint16_t, (_Float16)s0), hi = __builtin_bit_cast(uint16_t, (_Float16)s1);
        *reinterpret_cast<uint32_t *>(meta_scales16(meta) + idx) = lo | (hi << 16);
    } else {
        *reinterpret_cast<float2 *>(meta + idx) = make_float2(s0, s1);
    }
}

__device__ __forceinline__ float recip_or_zero(float s) { return s != 0.0f ? __builtin_amdgcn_rcpf(s) : 0.0f; }

__device__ __forceinline__ void load8(const float *p, float (&v)[8])
{
    *reinterpret_cast<float4 *>(&v[0]) = *reinterpret_cast<const float4 *>(p);
    *reinterpret_cast<float4 *>(&v[4]) = *reinterpret_cast<const float4 *>(p + 4);
}

// eight zero-points as they are kept (fp16, minima of fp16 inputs): one 16-byte read
__device__ __forceinline__ void load8_half(const uint16_t *p, uint32_t (&v)[4])
{
    const uint4 w = *reinterpret_cast<const uint4 *>(p);
    v[0] = w.x; v[1] = w.y; v[2] = w.z; v[3] = w.w;
}

// the value held by lane ^ 1 / lane ^ 2: exchanges inside a group of four lanes are done by the vector unit
// itself (data-parallel primitive, quad permutation), not through the LDS crossbar
__device__ __forceinline__ uint32_t from_lane_xor1(uint32_t x) { return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0xB1, 0xF, 0xF, true); }
__device__ __forceinline__ uint32_t from_lane_xor2(uint32_t x) { return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x4E, 0xF, 0xF, true); }

// Exchanges with lane ^ 16 and lane ^ 32, for symmetric uses only (min, max): the swap instructions exchange the
// odd rows of 16 lanes (the upper 32 lanes) of their first operand with the even rows (the lower 32 lanes) of their
// second.  Fed the same register twice, every lane ends up with its own value in one result and its partner's
// in the other (which is which depends on the lane).
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x2 pair_xor16(uint32_t x) { return __builtin_amdgcn_permlane16_swap(x, x, false, false); }
__device__ __forceinline__ u32x2 pair_xor32(uint32_t x) { return __builtin_amdgcn_permlane32_swap(x, x, false, false); }
// lane 7 - i of each 8 / lane 15 - i of each 16 (row mirrors): complete a reduction once the lanes of a quad agree
__device__ __forceinline__ uint32_t from_half_row_mirror(uint32_t x) { return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x141, 0xF, 0xF, true); }
__device__ __forceinline__ uint32_t from_row_mirror(uint32_t x) { return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, 0x140, 0xF, 0xF, true); }

// 16-bit half of the block-exponent word: exponent e of max = f * 2^e, f in [0.5, 1), biased by 32768
// (32768 itself for an all-constant block or an fp16 tensor)
__device__ __forceinline__ uint16_t biased_exponent(float wave_max)
{
    int e = 0;
    if (wave_max > 0.0f) (void)frexpf(wave_max, &e);
    return (uint16_t)(e + 32768);
}

// maximum over the wave of non-negative numbers (their bit patterns order like the numbers), in every lane
__device__ __forceinline__ float wave_max64(float xf)
{
    uint32_t x = __builtin_bit_cast(uint32_t, xf);
    x = max(x, from_lane_xor1(x));
    x = max(x, from_lane_xor2(x));
    x = max(x, from_half_row_mirror(x));
    x = max(x, from_row_mirror(x));
    u32x2 w = pair_xor16(x);
    x = max(w.x, w.y);
    w = pair_xor32(x);
    return __builtin_bit_cast(float, max(w.x, w.y));
}

// Row of channel ch in the transposed value tile.  Rows are 80 bytes (32 tokens + 16 bytes of padding); the
// low four bits of the row number are mixed with bits 3..6 of the channel so that both the 16 lanes that
// write one token chunk (channels 8*c16 + e) and the 16 lanes that read one (channels 16*m + n) fall on
// 16 different 16-byte bank groups.
__device__ __forceinline__ int value_row(int ch) { return (ch & 0x70) | ((ch ^ (ch >> 3)) & 15); }

// One wave per (tensor, block of 32 tokens, (b, h)); blockIdx.y = 0 keys, 1 values.  The statistics are
// taken in the arrangement the rows are loaded in (16 bytes = 8 channels of a token per lane), the tile
// goes through LDS, and each lane encodes exactly the 64 codes it stores.
template <int KB, int VB, bool NARROW>
__global__ __launch_bounds__(64) void quantize_blocks(QuantArgs a)
{
    const int lane = threadIdx.x;
    const int bh = blockIdx.x / a.n_blocks;
    const int blk = a.first_block + blockIdx.x % a.n_blocks;
    const bool values = blockIdx.y != 0;
    const int r = lane >> 4, c16 = lane & 15;
    const int n = lane & 15, kq = lane >> 4;

    // keys [token][channel] with rows of kD + 8 halves, or values [row of channel][token] with rows of 32 + 8 halves
    __shared__ __attribute__((aligned(16))) uint16_t tile[kD * (32 + 8)];
    __shared__ __attribute__((aligned(16))) float sc[kD], rsc[kD];            // scale (read only when a redo is needed), 1 / scale
    __shared__ __attribute__((aligned(16))) uint16_t zp[kD];                  // zero-point, fp16 as stored
    static_assert(kD * (32 + 8) >= 32 * (kD + 8), "one buffer serves both arrangements");

    // keys: lane = 16*r + c16 holds tokens r, r+4, .., r+28; values: tokens 8*r .. 8*r+7 (8 channels 8*c16.. each)
    const uint16_t *in = values ? a.v_in : a.k_in, *ring = values ? a.lv.vres : a.lv.kres;
    uint32_t x[8][4];
    if (blk * kG >= a.t_old) {
        // the whole block comes from the caller's tensor (always so in a prompt's first append): one row address, fixed steps
        const uint16_t *row0 = in + ((size_t)bh * a.n_in + (blk * kG - a.t_old) + (values ? 8 * r : r)) * kD + 8 * c16;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row0 + (values ? i : 4 * i) * kD));
            x[i][0] = w.x; x[i][1] = w.y; x[i][2] = w.z; x[i][3] = w.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const int pos = blk * kG + (values ? 8 * r + i : r + 4 * i);
            const uint4 w = *reinterpret_cast<const uint4 *>(token_row(in, ring, bh, pos, a.t_old, a.n_in, a.RC) + 8 * c16);
            x[i][0] = w.x; x[i][1] = w.y; x[i][2] = w.z; x[i][3] = w.w;
        }
    }
    float one;                                                   // 1.0, opaque to the compiler (see encode8)
    asm("s_mov_b32 %0, 1.0" : "=s"(one));
    const size_t blk_index = (size_t)bh * a.NB + blk;
    uint16_t *bexp16 = reinterpret_cast<uint16_t *>(a.lv.bexp + blk_index);    // [0] keys, [1] values

    if (!values) {
        // ================================================================= keys
        if constexpr (KB == 16) {
            uint8_t *dst = a.lv.kcode + blk_index * block_code_bytes(16);
#pragma unroll
            for (int i = 0; i < 8; i++)
                *reinterpret_cast<uint4 *>(dst + (r + 4 * i) * (kD * 2) + c16 * 16) = make_uint4(x[i][0], x[i][1], x[i][2], x[i][3]);
            if (lane == 0) bexp16[0] = 32768;
        } else {
            const bool kpt = a.lv.kpt != 0;                  // keys grouped per token over 32 channels, like the values
            float *meta = a.lv.kmeta + blk_index * meta_words(NARROW);
            float s_max = 0.0f;
            if (!kpt) {
                // min / max per channel over the lane's 8 tokens, then across the 4 lane rows by shuffles
                uint32_t mnp[4], mxp[4];
#pragma unroll
                for (int p = 0; p < 4; p++) { mnp[p] = x[0][p]; mxp[p] = x[0][p]; }
#pragma unroll
                for (int i = 1; i < 8; i++)
#pragma unroll
                    for (int p = 0; p < 4; p++) { mnp[p] = pk_min(mnp[p], x[i][p]); mxp[p] = pk_max(mxp[p], x[i][p]); }
#pragma unroll
                for (int p = 0; p < 4; p++) {
                    u32x2 w = pair_xor16(mnp[p]); mnp[p] = pk_min(w.x, w.y);
                    w = pair_xor16(mxp[p]); mxp[p] = pk_max(w.x, w.y);
                    w = pair_xor32(mnp[p]); mnp[p] = pk_min(w.x, w.y);
                    w = pair_xor32(mxp[p]); mxp[p] = pk_max(w.x, w.y);
                }
                // every lane row now holds the statistics of all 8 channels: row r finishes channels 2r and 2r + 1
                const uint32_t mn2 = plus_zero_pair(r == 0 ? mnp[0] : r == 1 ? mnp[1] : r == 2 ? mnp[2] : mnp[3]);
                const uint32_t mx2 = plus_zero_pair(r == 0 ? mxp[0] : r == 1 ? mxp[1] : r == 2 ? mxp[2] : mxp[3]);
                // the pair goes out as one store per array (scales, zero-points; LDS copies likewise)
                const int ch = 8 * c16 + 2 * r;
                float s2[2], r2[2];
#pragma unroll
                for (int h = 0; h < 2; h++) {
                    const float mn = half_bits_to_float((mn2 >> (16 * h)) & 0xffffu), mx = half_bits_to_float((mx2 >> (16 * h)) & 0xffffu);
                    s2[h] = stored_scale<NARROW>(scale_of(mn, mx, KB));
                    r2[h] = recip_or_zero(s2[h]);
                    s_max = fmaxf(s_max, s2[h]);
                }
                *reinterpret_cast<float2 *>(&sc[ch]) = make_float2(s2[0], s2[1]);
                *reinterpret_cast<float2 *>(&rsc[ch]) = make_float2(r2[0], r2[1]);
                *reinterpret_cast<uint32_t *>(&zp[ch]) = mn2;
                store_scale_pair<NARROW>(meta, ch, s2[0], s2[1]);
                *reinterpret_cast<uint32_t *>(meta_zeros(meta, NARROW) + ch) = mn2;
            } else {
                // min / max per token over the lane's 8 channels, then over the 4 lanes c16 = 4*gd .. 4*gd+3 of group gd;
                // metadata index 32*gd + token, as for values
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    const int t = r + 4 * i;
                    uint32_t mnp = pk_min(pk_min(x[i][0], x[i][1]), pk_min(x[i][2], x[i][3]));
                    uint32_t mxp = pk_max(pk_max(x[i][0], x[i][1]), pk_max(x[i][2], x[i][3]));
                    mnp = pk_min(mnp, from_lane_xor1(mnp)); mxp = pk_max(mxp, from_lane_xor1(mxp));
                    mnp = pk_min(mnp, from_lane_xor2(mnp)); mxp = pk_max(mxp, from_lane_xor2(mxp));
                    const float mn = plus_zero(fminf(half_bits_to_float(mnp & 0xffffu), half_bits_to_float(mnp >> 16)));
                    const float mx = plus_zero(fmaxf(half_bits_to_float(mxp & 0xffffu), half_bits_to_float(mxp >> 16)));
                    const float s = stored_scale<NARROW>(scale_of(mn, mx, KB));
                    s_max = fmaxf(s_max, s);
                    if ((c16 & 3) == 0) {
                        const int gd = c16 >> 2;
                        const uint16_t zb = float_to_half_bits_exact(mn);
                        sc[32 * gd + t] = s; zp[32 * gd + t] = zb; rsc[32 * gd + t] = recip_or_zero(s);
                        store_scale<NARROW>(meta, 32 * gd + t, s); meta_zeros(meta, NARROW)[32 * gd + t] = zb;
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < 8; i++)
                *reinterpret_cast<uint4 *>(&tile[(r + 4 * i) * (kD + 8) + 8 * c16]) = make_uint4(x[i][0], x[i][1], x[i][2], x[i][3]);
            s_max = wave_max64(s_max);
            if (lane == 0) bexp16[0] = biased_exponent(s_max);
            __syncthreads();
            // codes in the lane layout of kvq_layout.h: dword group m = 4*th + cb holds token 16*th + n, channels
            // 32*cb + 8*kq ..; the metadata of a channel set serves both token halves
            uint32_t dw[2 * KB];
#pragma unroll
            for (int cb = 0; cb < 4; cb++) {
                const int ch0 = 32 * cb + 8 * kq;
                uint32_t zw[4];
                float r8[8];
                if (!kpt) { load8_half(&zp[ch0], zw); load8(&rsc[ch0], r8); }
#pragma unroll
                for (int th = 0; th < 2; th++) {
                    const int m = 4 * th + cb, token = 16 * th + n;
                    const int gi = 32 * cb + token;               // per-token keys: one (s, z) for the 8 channels of this token and group
                    const uint4 xx = *reinterpret_cast<const uint4 *>(&tile[token * (kD + 8) + ch0]);
                    const uint32_t xw[4] = {xx.x, xx.y, xx.z, xx.w};
                    if (kpt) {
                        const uint32_t zb = zp[gi];
                        const float rr = rsc[gi];
#pragma unroll
                        for (int e = 0; e < 4; e++) zw[e] = zb | (zb << 16);
#pragma unroll
                        for (int e = 0; e < 8; e++) r8[e] = rr;
                    }
                    float d[8], c8[8];
                    if (encode8<KB, NARROW>(xw, zw, r8, one, d, c8)) {
                        float s8[8];
                        if (!kpt) {
                            load8(&sc[ch0], s8);
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; e++) s8[e] = sc[gi];
                        }
                        redo8<KB>(d, s8, c8);
                    }
                    pack8<KB>(c8, m, dw);
                }
            }
            uint8_t *dst = a.lv.kcode + blk_index * block_code_bytes(KB);
#pragma unroll
            for (int c = 0; c < KB / 2; c++)
                __builtin_nontemporal_store(u32x4{dw[4 * c], dw[4 * c + 1], dw[4 * c + 2], dw[4 * c + 3]}, reinterpret_cast<u32x4 *>(dst + c * 1024 + lane * 16));
        }
    } else {
        // ================================================================= values
        if constexpr (VB == 16) {
            uint8_t *dst = a.lv.vcode + blk_index * block_code_bytes(16);
#pragma unroll
            for (int i = 0; i < 8; i++)
                *reinterpret_cast<uint4 *>(dst + (8 * r + i) * (kD * 2) + c16 * 16) = make_uint4(x[i][0], x[i][1], x[i][2], x[i][3]);
            if (lane == 0) bexp16[1] = 32768;
        } else {
            float *meta = a.lv.vmeta + blk_index * meta_words(NARROW);
            float s_max = 0.0f;
            // min / max over the lane's 8 channels, then over the 4 lanes c16 = 4*gd .. 4*gd+3 of group gd (fp16 pairs:
            // the two halves are merged below)
            uint32_t mnp[8], mxp[8];
#pragma unroll
            for (int i = 0; i < 8; i++) {
                mnp[i] = pk_min(pk_min(x[i][0], x[i][1]), pk_min(x[i][2], x[i][3]));
                mxp[i] = pk_max(pk_max(x[i][0], x[i][1]), pk_max(x[i][2], x[i][3]));
                mnp[i] = pk_min(mnp[i], from_lane_xor1(mnp[i])); mxp[i] = pk_max(mxp[i], from_lane_xor1(mxp[i]));
                mnp[i] = pk_min(mnp[i], from_lane_xor2(mnp[i])); mxp[i] = pk_max(mxp[i], from_lane_xor2(mxp[i]));
            }
            // the 4 lanes of a group hold the same 8 results: lane q = c16 & 3 finishes tokens 2q and 2q + 1 of its row,
            // a pair that goes out as one store per array
            const int q4 = c16 & 3, gd = c16 >> 2;
            const int t0 = 32 * gd + 8 * r + 2 * q4;
            float s2[2], r2[2];
            uint32_t z2 = 0;
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const uint32_t mnb = q4 == 0 ? mnp[h] : q4 == 1 ? mnp[2 + h] : q4 == 2 ? mnp[4 + h] : mnp[6 + h];
                const uint32_t mxb = q4 == 0 ? mxp[h] : q4 == 1 ? mxp[2 + h] : q4 == 2 ? mxp[4 + h] : mxp[6 + h];
                const float mn = plus_zero(fminf(half_bits_to_float(mnb & 0xffffu), half_bits_to_float(mnb >> 16)));
                const float mx = plus_zero(fmaxf(half_bits_to_float(mxb & 0xffffu), half_bits_to_float(mxb >> 16)));
                s2[h] = stored_scale<NARROW>(scale_of(mn, mx, VB));
                r2[h] = recip_or_zero(s2[h]);
                s_max = fmaxf(s_max, s2[h]);
                z2 |= (uint32_t)float_to_half_bits_exact(mn) << (16 * h);
            }
            *reinterpret_cast<float2 *>(&sc[t0]) = make_float2(s2[0], s2[1]);
            *reinterpret_cast<float2 *>(&rsc[t0]) = make_float2(r2[0], r2[1]);
            *reinterpret_cast<uint32_t *>(&zp[t0]) = z2;
            store_scale_pair<NARROW>(meta, t0, s2[0], s2[1]);
            *reinterpret_cast<uint32_t *>(meta_zeros(meta, NARROW) + t0) = z2;
            // 8 x 8 transpose in registers: channel 8*c16 + e gets its 8 tokens as one 16-byte chunk
            const int krow = (c16 & 7) | (((c16 ^ (c16 >> 3)) & 1) << 3);      // value_row(8*c16 + e) = (c16 >> 1) << 4 | (krow ^ e)
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
                const uint4 w = make_uint4(__builtin_amdgcn_perm(x[1][e >> 1], x[0][e >> 1], sel), __builtin_amdgcn_perm(x[3][e >> 1], x[2][e >> 1], sel),
                                           __builtin_amdgcn_perm(x[5][e >> 1], x[4][e >> 1], sel), __builtin_amdgcn_perm(x[7][e >> 1], x[6][e >> 1], sel));
                const int row = ((c16 >> 1) << 4) | (krow ^ e);
                *reinterpret_cast<uint4 *>(&tile[row * (32 + 8) + 8 * r]) = w;
            }
            s_max = wave_max64(s_max);
            if (lane == 0) bexp16[1] = biased_exponent(s_max);
            __syncthreads();
            uint32_t dw[2 * VB];
            const int nrow = (n ^ (n >> 3)) & 15;                               // value_row(16*m + n) = m << 4 | (nrow ^ 2*m)
#pragma unroll
            for (int gd = 0; gd < 4; gd++) {
                // the lane's tokens 8*kq .. 8*kq + 7 of channel group gd: one set of metadata for two dword groups
                uint32_t zw[4];
                float r8[8];
                load8_half(&zp[32 * gd + 8 * kq], zw); load8(&rsc[32 * gd + 8 * kq], r8);
#pragma unroll
                for (int j = 0; j < 2; j++) {
                    const int m = 2 * gd + j, row = (m << 4) | (nrow ^ ((2 * m) & 15));
                    const uint4 xx = *reinterpret_cast<const uint4 *>(&tile[row * (32 + 8) + 8 * kq]);
                    const uint32_t xw[4] = {xx.x, xx.y, xx.z, xx.w};
                    float d[8], c8[8];
                    if (encode8<VB, NARROW>(xw, zw, r8, one, d, c8)) {
                        float s8[8];
                        load8(&sc[32 * gd + 8 * kq], s8);
                        redo8<VB>(d, s8, c8);
                    }
                    pack8<VB>(c8, m, dw);
                }
            }
            uint8_t *dst = a.lv.vcode + blk_index * block_code_bytes(VB);
#pragma unroll
            for (int c = 0; c < VB / 2; c++)
                __builtin_nontemporal_store(u32x4{dw[4 * c], dw[4 * c + 1], dw[4 * c + 2], dw[4 * c + 3]}, reinterpret_cast<u32x4 *>(dst + c * 1024 + lane * 16));
        }
    }
}

// New tokens that stay in the fp16 window: input rows -> ring slots.  16 lanes per token row.
__global__ __launch_bounds__(256) void window_copy(ResidualCopyArgs a)
{
    const int n_tok = a.pos1 - a.pos0;
    const long long item = (long long)blockIdx.x * 16 + (threadIdx.x >> 4);   // (bh, token) pairs
    if (item >= (long long)a.BH * n_tok) return;
    const int bh = (int)(item / n_tok), pos = a.pos0 + (int)(item % n_tok), c16 = threadIdx.x & 15;
    const size_t src = ((size_t)bh * a.n_in + (pos - a.t_old)) * kD + 8 * c16;
    const size_t dst = ((size_t)bh * a.RC + pos % a.RC) * kD + 8 * c16;
    *reinterpret_cast<uint4 *>(a.lv.kres + dst) = *reinterpret_cast<const uint4 *>(a.k_in + src);
    *reinterpret_cast<uint4 *>(a.lv.vres + dst) = *reinterpret_cast<const uint4 *>(a.v_in + src);
}

// ---- canonical export (debug / test path; one thread per output element group)

template <int BITS>
__device__ __forceinline__ uint32_t fetch_code(const uint8_t *block, int lane, int ci)
{
    int dw, sh;
    if (BITS == 8) { dw = ci / 4; sh = 8 * (ci % 4); }
    else if (BITS == 4) { dw = ci / 8; sh = 4 * (((ci % 8) >> 1) + 4 * (ci & 1)); }
    else { dw = ci / 16; sh = 2 * (4 * ((ci / 8) & 1) + ((ci % 8) >> 1) + 8 * (ci & 1)); }
    const uint32_t w = *reinterpret_cast<const uint32_t *>(block + dword_offset(lane, dw));
    return (w >> sh) & ((1u << BITS) - 1u);
}

__device__ __forceinline__ uint32_t fetch_code_rt(int bits, const uint8_t *block, int lane, int ci)
{
    return bits == 8 ? fetch_code<8>(block, lane, ci) : bits == 4 ? fetch_code<4>(block, lane, ci) : fetch_code<2>(block, lane, ci);
}

// keys grouped per token: one thread per canonical output byte [bh][token][byte], the 128 channels of a token
__global__ void export_key_codes_per_token(ExportArgs a)
{
    const int kb = a.lv.kbits;
    const int tbytes = kD * kb / 8, per_byte = 8 / kb;
    const long long total = (long long)a.BH * a.n_packed * tbytes;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int by = (int)(idx % tbytes);
    const int tok = (int)((idx / tbytes) % a.n_packed);
    const int bh = (int)(idx / ((long long)tbytes * a.n_packed));
    const uint8_t *block = a.lv.kcode + ((size_t)bh * a.NB + tok / kG) * block_code_bytes(kb);
    const int t = tok % kG;
    uint32_t v = 0;
    for (int j = 0; j < per_byte; j++) {
        const int d = by * per_byte + j;
        v |= fetch_code_rt(kb, block, key_lane(t, d), key_ci(t, d)) << (j * kb);
    }
    a.k_codes[idx] = (uint8_t)v;
}

// keys: one thread per canonical output byte [bh][g][d][byte]
__global__ void export_key_codes(ExportArgs a)
{
    const int kb = a.lv.kbits;
    const int gbytes = kG * kb / 8, per_byte = 8 / kb;
    const long long total = (long long)a.BH * (a.n_packed / kG) * kD * gbytes;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int by = (int)(idx % gbytes);
    const int d = (int)((idx / gbytes) % kD);
    const int g = (int)((idx / ((long long)gbytes * kD)) % (a.n_packed / kG));
    const int bh = (int)(idx / ((long long)gbytes * kD * (a.n_packed / kG)));
    const uint8_t *block = a.lv.kcode + ((size_t)bh * a.NB + g) * block_code_bytes(kb);
    uint32_t v = 0;
    for (int j = 0; j < per_byte; j++) {
        const int t = by * per_byte + j;
        v |= fetch_code_rt(kb, block, key_lane(t, d), key_ci(t, d)) << (j * kb);
    }
    a.k_codes[idx] = (uint8_t)v;
}

// values: one thread per canonical output byte [bh][token][byte]
__global__ void export_value_codes(ExportArgs a)
{
    const int vb = a.lv.vbits;
    const int tbytes = kD * vb / 8, per_byte = 8 / vb;
    const long long total = (long long)a.BH * a.n_packed * tbytes;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int by = (int)(idx % tbytes);
    const int tok = (int)((idx / tbytes) % a.n_packed);
    const int bh = (int)(idx / ((long long)tbytes * a.n_packed));
    const uint8_t *block = a.lv.vcode + ((size_t)bh * a.NB + tok / kG) * block_code_bytes(vb);
    const int t = tok % kG;
    uint32_t v = 0;
    for (int j = 0; j < per_byte; j++) {
        const int d = by * per_byte + j;
        v |= fetch_code_rt(vb, block, val_lane(t, d), val_ci(t, d)) << (j * vb);
    }
    a.v_codes[idx] = (uint8_t)v;
}

// metadata: keys [bh][g][d], values [bh][token][gd]; one thread per element
__global__ void export_meta(ExportArgs a, int which)   // 0 = keys, 1 = values
{
    const long long total = (long long)a.BH * (a.n_packed / kG) * kD;   // same element count for both
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int within = (int)(idx % kD);
    const int g = (int)((idx / kD) % (a.n_packed / kG));
    const int bh = (int)(idx / ((long long)kD * (a.n_packed / kG)));
    const bool narrow = a.lv.narrow != 0;
    const float *meta = (which == 0 ? a.lv.kmeta : a.lv.vmeta) + ((size_t)bh * a.NB + g) * meta_words(narrow);
    float *so = which == 0 ? a.k_scale : a.v_scale, *zo = which == 0 ? a.k_zero : a.v_zero;
    // canonical value (and per-token key) metadata is [token][group]; the device keeps [group][token]
    const int src = which == 0 && !a.lv.kpt ? within : 32 * (within & 3) + (within >> 2);
    if (so) so[idx] = narrow ? half_bits_to_float(meta_scales16(meta)[src]) : meta[src];
    if (zo) zo[idx] = half_bits_to_float(meta_zeros(meta, narrow)[src]);
}

// fp16 tensors: rows [bh][token][128]; one thread per 16 bytes.  which: 0/1 = 16-bit keys / values of the
// quantized region, 2/3 = window keys / values.
__global__ void export_rows(ExportArgs a, int which)
{
    const int n_tok = which < 2 ? a.n_packed : a.n_res;
    const long long total = (long long)a.BH * n_tok * 16;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int c16 = (int)(idx % 16);
    const int tok = (int)((idx / 16) % n_tok);
    const int bh = (int)(idx / (16LL * n_tok));
    const uint16_t *src;
    uint16_t *dst;
    if (which < 2) {
        const uint8_t *base = which == 0 ? a.lv.kcode : a.lv.vcode;
        src = reinterpret_cast<const uint16_t *>(base + ((size_t)bh * a.NB * kG + tok) * (kD * 2));
        dst = reinterpret_cast<uint16_t *>(which == 0 ? a.k_codes : a.v_codes);
    } else {
        const uint16_t *ring = which == 2 ? a.lv.kres : a.lv.vres;
        src = ring + ((size_t)bh * a.RC + (a.n_packed + tok) % a.RC) * kD;
        dst = which == 2 ? a.k_res : a.v_res;
    }
    *reinterpret_cast<uint4 *>(dst + ((size_t)bh * n_tok + tok) * kD + 8 * c16) = *reinterpret_cast<const uint4 *>(src + 8 * c16);
}

template <int KB, bool NARROW>
hipError_t launch_quantize_vb(const QuantArgs &a, hipStream_t s)
{
    const dim3 grid((unsigned)a.n_blocks * (unsigned)a.BH, 2), block(64);
    switch (a.lv.vbits) {
    case 2: hipLaunchKernelGGL((quantize_blocks<KB, 2, NARROW>), grid, block, 0, s, a); break;
    case 4: hipLaunchKernelGGL((quantize_blocks<KB, 4, NARROW>), grid, block, 0, s, a); break;
    case 8: hipLaunchKernelGGL((quantize_blocks<KB, 8, NARROW>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((quantize_blocks<KB, 16, NARROW>), grid, block, 0, s, a); break;
    }
    return hipGetLastError();
}

template <bool NARROW>
hipError_t launch_quantize_kb(const QuantArgs &a, hipStream_t s)
{
    switch (a.lv.kbits) {
    case 2: return launch_quantize_vb<2, NARROW>(a, s);
    case 4: return launch_quantize_vb<4, NARROW>(a, s);
    case 8: return launch_quantize_vb<8, NARROW>(a, s);
    default: return launch_quantize_vb<16, NARROW>(a, s);
    }
}

unsigned blocks_for(long long total, int threads) { return (unsigned)((total + threads - 1) / threads); }

}  // namespace

hipError_t launch_quantize(const QuantArgs &a, hipStream_t s)
{
    if (a.n_blocks < 1 || a.BH < 1) return hipSuccess;
    if ((long long)a.n_blocks * a.BH > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    return a.lv.narrow ? launch_quantize_kb<true>(a, s) : launch_quantize_kb<false>(a, s);
}

hipError_t launch_residual_copy(const ResidualCopyArgs &a, hipStream_t s)
{
    const long long items = (long long)a.BH * (a.pos1 - a.pos0);
    if (items < 1) return hipSuccess;
    hipLaunchKernelGGL(window_copy, dim3(blocks_for(items, 16)), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_export(const ExportArgs &a, hipStream_t s)
{
    const int T = 256;
    if (a.n_packed > 0) {
        const long long meta_elems = (long long)a.BH * (a.n_packed / kG) * kD;
        if (a.lv.kbits < 16) {
            if (a.k_codes)
                hipLaunchKernelGGL(a.lv.kpt ? export_key_codes_per_token : export_key_codes,
                                   dim3(blocks_for(meta_elems * (kG * a.lv.kbits / 8), T)), dim3(T), 0, s, a);
            if (a.k_scale || a.k_zero) hipLaunchKernelGGL(export_meta, dim3(blocks_for(meta_elems, T)), dim3(T), 0, s, a, 0);
        } else if (a.k_codes) {
            hipLaunchKernelGGL(export_rows, dim3(blocks_for((long long)a.BH * a.n_packed * 16, T)), dim3(T), 0, s, a, 0);
        }
        if (a.lv.vbits < 16) {
            if (a.v_codes)
                hipLaunchKernelGGL(export_value_codes, dim3(blocks_for((long long)a.BH * a.n_packed * (kD * a.lv.vbits / 8), T)), dim3(T), 0, s, a);
            if (a.v_scale || a.v_zero) hipLaunchKernelGGL(export_meta, dim3(blocks_for(meta_elems, T)), dim3(T), 0, s, a, 1);
        } else if (a.v_codes) {
            hipLaunchKernelGGL(export_rows, dim3(blocks_for((long long)a.BH * a.n_packed * 16, T)), dim3(T), 0, s, a, 1);
        }
    }
    if (a.n_res > 0) {
        if (a.k_res) hipLaunchKernelGGL(export_rows, dim3(blocks_for((long long)a.BH * a.n_res * 16, T)), dim3(T), 0, s, a, 2);
        if (a.v_res) hipLaunchKernelGGL(export_rows, dim3(blocks_for((long long)a.BH * a.n_res * 16, T)), dim3(T), 0, s, a, 3);
    }
    return hipGetLastError();
}

}  // namespace kvq
