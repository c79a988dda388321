// Device-side storage layout of the quantized KV cache (gfx950, wave64).
//
// The quantized part of a layer is stored in blocks of 32 tokens x 128 channels
// per (batch, kv head).  Inside a block the codes are arranged for the lane
// mapping of the 16x16x32 matrix-core instruction, with lane = 16*kq + n
// (n = lane & 15, kq = lane >> 4) owning 64 codes, numbered ci = 8*m + e:
//
//   keys   (contraction over channels):  m = 4*th + cb
//            token   = 16*th + n
//            channel = 32*cb + 8*kq + e
//   values (contraction over tokens):    m = cblk
//            token   = 8*kq + e
//            channel = 16*cblk + n
//
// A lane's 64 codes occupy 16 * bits / 8 ... i.e. 8*bits bytes, stored as bits/2
// chunks of 16 bytes; chunk c of lane l sits at block_base + c*1024 + l*16, so a
// wave reads 1 KiB contiguously per load instruction.  Within the lane's dwords:
//   8 bit : code ci in dword ci/4,  bits [8*(ci%4), +8)
//   4 bit : dword m, nibble (e>>1) + 4*(e&1)   (nibbles k and k+4 form an fp16 pair)
//   2 bit : dword m/2, field 4*(m&1) + (e>>1) + 8*(e&1)
//
// Metadata of a block: 128 fp32 scales, then 128 zero-points as fp16 (768 bytes).  A zero-point
// is the minimum of a group of fp16 inputs, so it is an fp16 number and the narrow store is exact.
// In the narrow-metadata variant the scales are fp16 as well (512 bytes per block).
//   keys  : index = channel              (per channel over the block's 32 tokens)
//   values: index = 32*(channel/32) + token (per token over 32 channels)
//
// 16-"bit" tensors keep fp16 rows [token][128] (no metadata); a block is 8 KiB.
#pragma once
#include <stdint.h>

namespace kvq {

constexpr int kD = 128;       // head dimension
constexpr int kG = 32;        // group size: tokens per key group, channels per value group
// a block's metadata in dwords: scales, then zero-points (fp16); narrow = scales as fp16 too
__host__ __device__ constexpr int meta_words(bool narrow) { return narrow ? 128 : 192; }

__host__ __device__ constexpr int block_code_bytes(int bits) { return bits == 16 ? 32 * kD * 2 : 512 * bits; }
__host__ __device__ constexpr int block_meta_bytes(int bits, bool narrow) { return bits == 16 ? 0 : 4 * meta_words(narrow); }

// dword index (0 .. 2*bits-1) and bit shift of code ci (0..63) inside a lane's codes
template <int BITS>
__host__ __device__ constexpr int code_dword(int ci)
{
    return BITS == 8 ? ci / 4 : BITS == 4 ? ci / 8 : ci / 16;
}
template <int BITS>
__host__ __device__ constexpr int code_shift(int ci)
{
    return BITS == 8 ? 8 * (ci % 4)
         : BITS == 4 ? 4 * (((ci % 8) >> 1) + 4 * (ci & 1))
                     : 2 * (4 * ((ci / 8) & 1) + ((ci % 8) >> 1) + 8 * (ci & 1));
}
// byte offset of dword dw of lane l inside a block
__host__ __device__ constexpr int dword_offset(int lane, int dw) { return (dw / 4) * 1024 + lane * 16 + (dw % 4) * 4; }

// (token, channel) of code ci of lane l
__host__ __device__ constexpr int key_token(int lane, int ci) { return 16 * (ci / 32) + (lane & 15); }
__host__ __device__ constexpr int key_channel(int lane, int ci) { return 32 * ((ci / 8) & 3) + 8 * (lane >> 4) + (ci & 7); }
__host__ __device__ constexpr int val_token(int lane, int ci) { return 8 * (lane >> 4) + (ci & 7); }
__host__ __device__ constexpr int val_channel(int lane, int ci) { return 16 * (ci / 8) + (lane & 15); }

// inverse maps: which lane / code index holds (token t in 0..31, channel d in 0..127)
__host__ __device__ constexpr int key_lane(int t, int d) { return 16 * ((d & 31) >> 3) + (t & 15); }
__host__ __device__ constexpr int key_ci(int t, int d) { return 8 * (4 * (t >> 4) + (d >> 5)) + (d & 7); }
__host__ __device__ constexpr int val_lane(int t, int d) { return 16 * (t >> 3) + (d & 15); }
__host__ __device__ constexpr int val_ci(int t, int d) { return 8 * (d >> 4) + (t & 7); }

// zero-points (fp16 bit patterns) and, in the narrow variant, scales (fp16 bit patterns) of the metadata
// block that starts at `meta`
__host__ __device__ inline const uint16_t *meta_zeros(const float *meta, bool narrow) { return reinterpret_cast<const uint16_t *>(meta) + (narrow ? 128 : 256); }
__host__ __device__ inline uint16_t *meta_zeros(float *meta, bool narrow) { return reinterpret_cast<uint16_t *>(meta) + (narrow ? 128 : 256); }
__host__ __device__ inline const uint16_t *meta_scales16(const float *meta) { return reinterpret_cast<const uint16_t *>(meta); }
__host__ __device__ inline uint16_t *meta_scales16(float *meta) { return reinterpret_cast<uint16_t *>(meta); }

}  // namespace kvq
