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

template <int BITS>
__device__ __forceinline__ uint32_t encode(float x, float s, float z)
{
    float t = s != 0.0f ? __fdiv_rn(x - z, s) : 0.0f;
    float r = rintf(t);
    r = fminf(fmaxf(r, 0.0f), (float)((1 << BITS) - 1));
    return (uint32_t)r;
}

__device__ __forceinline__ float scale_of(float mn, float mx, int bits)
{
    return __fdiv_rn(mx - mn, (float)((1 << bits) - 1));
}

// One wave per (block of 32 tokens, (b, h)).  Lane = 16*r + c16 loads 8 channels
// (8*c16 ..) of tokens r, r+4, .., r+28 for both tensors.
template <int KB, int VB>
__global__ __launch_bounds__(64) void quantize_blocks(QuantArgs a)
{
    const int lane = threadIdx.x;
    const int bh = blockIdx.x / a.n_blocks;
    const int blk = a.first_block + blockIdx.x % a.n_blocks;
    const int r = lane >> 4, c16 = lane & 15;
    const int n = lane & 15, kq = lane >> 4;

    __shared__ __attribute__((aligned(16))) uint16_t tk[32][kD + 8];     // keys [token][channel]
    __shared__ __attribute__((aligned(16))) uint16_t tvT[kD][32 + 8];    // values [channel][token]
    __shared__ __attribute__((aligned(16))) float ks[kD], kz[kD], vs[kD], vz[kD];

    uint32_t kx[8][4], vx[8][4];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const int pos = blk * kG + r + 4 * i;
        const uint4 kk = *reinterpret_cast<const uint4 *>(token_row(a.k_in, a.lv.kres, bh, pos, a.t_old, a.n_in, a.RC) + 8 * c16);
        const uint4 vv = *reinterpret_cast<const uint4 *>(token_row(a.v_in, a.lv.vres, bh, pos, a.t_old, a.n_in, a.RC) + 8 * c16);
        kx[i][0] = kk.x; kx[i][1] = kk.y; kx[i][2] = kk.z; kx[i][3] = kk.w;
        vx[i][0] = vv.x; vx[i][1] = vv.y; vx[i][2] = vv.z; vx[i][3] = vv.w;
    }
    const size_t blk_index = (size_t)bh * a.NB + blk;
    float ks_max = 0.0f, vs_max = 0.0f;     // largest scale of the block, for the matrix-core kernel's operand scaling

    // ---- keys
    if constexpr (KB == 16) {
        uint8_t *dst = a.lv.kcode + blk_index * block_code_bytes(16);
#pragma unroll
        for (int i = 0; i < 8; i++)
            *reinterpret_cast<uint4 *>(dst + (r + 4 * i) * (kD * 2) + c16 * 16) = make_uint4(kx[i][0], kx[i][1], kx[i][2], kx[i][3]);
    } else {
        // min / max per channel over the lane's 8 tokens, then across the 4 lane rows by shuffles
        float mn[8], mx[8];
#pragma unroll
        for (int e = 0; e < 8; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }
#pragma unroll
        for (int i = 0; i < 8; i++)
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const float x = half_bits_to_float((kx[i][e >> 1] >> (16 * (e & 1))) & 0xffffu);
                mn[e] = fminf(mn[e], x);
                mx[e] = fmaxf(mx[e], x);
            }
#pragma unroll
        for (int e = 0; e < 8; e++) {
            mn[e] = fminf(mn[e], __shfl_xor(mn[e], 16)); mx[e] = fmaxf(mx[e], __shfl_xor(mx[e], 16));
            mn[e] = fminf(mn[e], __shfl_xor(mn[e], 32)); mx[e] = fmaxf(mx[e], __shfl_xor(mx[e], 32));
        }
        float *meta = a.lv.kmeta + blk_index * kMetaWords;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const float s = scale_of(mn[e], mx[e], KB);
            ks_max = fmaxf(ks_max, s);
            if (r == 0) {
                ks[8 * c16 + e] = s; kz[8 * c16 + e] = mn[e];
                meta[8 * c16 + e] = s; meta_zeros(meta)[8 * c16 + e] = float_to_half_bits_exact(mn[e]);
            }
        }
#pragma unroll
        for (int i = 0; i < 8; i++)
            *reinterpret_cast<uint4 *>(&tk[r + 4 * i][8 * c16]) = make_uint4(kx[i][0], kx[i][1], kx[i][2], kx[i][3]);
    }

    // ---- values
    if constexpr (VB == 16) {
        uint8_t *dst = a.lv.vcode + blk_index * block_code_bytes(16);
#pragma unroll
        for (int i = 0; i < 8; i++)
            *reinterpret_cast<uint4 *>(dst + (r + 4 * i) * (kD * 2) + c16 * 16) = make_uint4(vx[i][0], vx[i][1], vx[i][2], vx[i][3]);
    } else {
        float *meta = a.lv.vmeta + blk_index * kMetaWords;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const int t = r + 4 * i;
            float mn = INFINITY, mx = -INFINITY;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const uint32_t hb = (vx[i][e >> 1] >> (16 * (e & 1))) & 0xffffu;
                const float x = half_bits_to_float(hb);
                mn = fminf(mn, x);
                mx = fmaxf(mx, x);
                tvT[8 * c16 + e][t] = (uint16_t)hb;
            }
            // the 4 lanes c16 = 4*gd .. 4*gd+3 hold the 32 channels of group gd
            mn = fminf(mn, __shfl_xor(mn, 1)); mx = fmaxf(mx, __shfl_xor(mx, 1));
            mn = fminf(mn, __shfl_xor(mn, 2)); mx = fmaxf(mx, __shfl_xor(mx, 2));
            const float s = scale_of(mn, mx, VB);
            vs_max = fmaxf(vs_max, s);
            if ((c16 & 3) == 0) {
                const int gd = c16 >> 2;
                vs[32 * gd + t] = s; vz[32 * gd + t] = mn;
                meta[32 * gd + t] = s; meta_zeros(meta)[32 * gd + t] = float_to_half_bits_exact(mn);
            }
        }
    }
    if constexpr (KB < 16 || VB < 16) {
#pragma unroll
        for (int sft = 1; sft < 64; sft <<= 1) {
            ks_max = fmaxf(ks_max, __shfl_xor(ks_max, sft));
            vs_max = fmaxf(vs_max, __shfl_xor(vs_max, sft));
        }
        if (lane == 0) {
            int ek = 0, ev = 0;                       // max = f * 2^e with f in [0.5, 1); 0 for an all-constant block
            if (ks_max > 0.0f) (void)frexpf(ks_max, &ek);
            if (vs_max > 0.0f) (void)frexpf(vs_max, &ev);
            a.lv.bexp[blk_index] = ((uint32_t)(ek + 32768) & 0xffffu) | ((uint32_t)(ev + 32768) << 16);
        }
    }
    __syncthreads();

    // ---- key codes in the lane layout of kvq_layout.h
    if constexpr (KB < 16) {
        uint32_t dw[2 * KB];
#pragma unroll
        for (int i = 0; i < 2 * KB; i++) dw[i] = 0;
#pragma unroll
        for (int m = 0; m < 8; m++) {
            const int token = 16 * (m >> 2) + n, ch0 = 32 * (m & 3) + 8 * kq;
            const uint4 xx = *reinterpret_cast<const uint4 *>(&tk[token][ch0]);
            const uint32_t xw[4] = {xx.x, xx.y, xx.z, xx.w};
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const float x = half_bits_to_float((xw[e >> 1] >> (16 * (e & 1))) & 0xffffu);
                const uint32_t c = encode<KB>(x, ks[ch0 + e], kz[ch0 + e]);
                dw[code_dword<KB>(8 * m + e)] |= c << code_shift<KB>(8 * m + e);
            }
        }
        uint8_t *dst = a.lv.kcode + blk_index * block_code_bytes(KB);
#pragma unroll
        for (int c = 0; c < KB / 2; c++)
            *reinterpret_cast<uint4 *>(dst + c * 1024 + lane * 16) = make_uint4(dw[4 * c], dw[4 * c + 1], dw[4 * c + 2], dw[4 * c + 3]);
    }
    // ---- value codes
    if constexpr (VB < 16) {
        uint32_t dw[2 * VB];
#pragma unroll
        for (int i = 0; i < 2 * VB; i++) dw[i] = 0;
#pragma unroll
        for (int m = 0; m < 8; m++) {
            const int ch = 16 * m + n, gd = m >> 1;
            const uint4 xx = *reinterpret_cast<const uint4 *>(&tvT[ch][8 * kq]);
            const uint32_t xw[4] = {xx.x, xx.y, xx.z, xx.w};
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const int t = 8 * kq + e;
                const float x = half_bits_to_float((xw[e >> 1] >> (16 * (e & 1))) & 0xffffu);
                const uint32_t c = encode<VB>(x, vs[32 * gd + t], vz[32 * gd + t]);
                dw[code_dword<VB>(8 * m + e)] |= c << code_shift<VB>(8 * m + e);
            }
        }
        uint8_t *dst = a.lv.vcode + blk_index * block_code_bytes(VB);
#pragma unroll
        for (int c = 0; c < VB / 2; c++)
            *reinterpret_cast<uint4 *>(dst + c * 1024 + lane * 16) = make_uint4(dw[4 * c], dw[4 * c + 1], dw[4 * c + 2], dw[4 * c + 3]);
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
    const float *meta = (which == 0 ? a.lv.kmeta : a.lv.vmeta) + ((size_t)bh * a.NB + g) * kMetaWords;
    float *so = which == 0 ? a.k_scale : a.v_scale, *zo = which == 0 ? a.k_zero : a.v_zero;
    // canonical value metadata is [token][group]; the device keeps [group][token]
    const int src = which == 0 ? within : 32 * (within & 3) + (within >> 2);
    if (so) so[idx] = meta[src];
    if (zo) zo[idx] = half_bits_to_float(meta_zeros(meta)[src]);
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

template <int KB>
hipError_t launch_quantize_vb(const QuantArgs &a, hipStream_t s)
{
    const dim3 grid((unsigned)a.n_blocks * (unsigned)a.BH), block(64);
    switch (a.lv.vbits) {
    case 2: hipLaunchKernelGGL((quantize_blocks<KB, 2>), grid, block, 0, s, a); break;
    case 4: hipLaunchKernelGGL((quantize_blocks<KB, 4>), grid, block, 0, s, a); break;
    case 8: hipLaunchKernelGGL((quantize_blocks<KB, 8>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((quantize_blocks<KB, 16>), grid, block, 0, s, a); break;
    }
    return hipGetLastError();
}

unsigned blocks_for(long long total, int threads) { return (unsigned)((total + threads - 1) / threads); }

}  // namespace

hipError_t launch_quantize(const QuantArgs &a, hipStream_t s)
{
    if (a.n_blocks < 1 || a.BH < 1) return hipSuccess;
    if ((long long)a.n_blocks * a.BH > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    switch (a.lv.kbits) {
    case 2: return launch_quantize_vb<2>(a, s);
    case 4: return launch_quantize_vb<4>(a, s);
    case 8: return launch_quantize_vb<8>(a, s);
    default: return launch_quantize_vb<16>(a, s);
    }
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
                hipLaunchKernelGGL(export_key_codes, dim3(blocks_for(meta_elems * (kG * a.lv.kbits / 8), T)), dim3(T), 0, s, a);
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
