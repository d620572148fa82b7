// Device-side helpers shared by the kernels of libtw: 16-byte bf16 vectors,
// range-checked buffer access, bf16 <-> fp32, and the lane-group sum.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tw {

// 16 bytes = 8 bf16, the unit of every load and store
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Raw buffer descriptors: byte-addressed, range-checked against num_records, so
// a lane whose offset is past the end reads zeros and its store is dropped.
// That is what handles ragged tails (rows past N, columns past H) in the kernels.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, static_cast<int>(bytes), 0x00020000);
}
static constexpr uint32_t kOutOfRange = 0xFFFFFFF0u;
static constexpr int kStreamPolicy = 2;  // loads, "nt": streamed once, do not keep in cache
// Stores, "sc1": measured against "nt" and the default on MI355X it is 5-9 %
// faster for whole-device launches of 0.3-0.8 GB, 2-3 % faster when a GEMM reads
// the output next, the same under a CU budget and 1-2 % slower beyond 1 GB.
static constexpr int kStorePolicy = 16;

__device__ __forceinline__ u32x4 ld(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, kStreamPolicy);
}
// `streamed` (a constant in every kernel that stores: each is built both ways,
// a choice at run time costs the small launches 2 %): the outputs of the call are
// larger than the 256 MiB last-level cache; they are then stored "nt" like the
// loads: 1-2 % faster from 8K rows of 8192 on, and a GEMM that runs next to the
// kernel or after it keeps more of its operands cached (a layer boundary of 16K
// tokens: 4-5 % faster); at 4K rows "sc1" is 4 % ahead.
__device__ __forceinline__ void st(__amdgpu_buffer_rsrc_t r, uint32_t off, u32x4 v, bool streamed)
{
    if (streamed) __builtin_amdgcn_raw_buffer_store_b128(v, r, off, 0, kStreamPolicy);
    else __builtin_amdgcn_raw_buffer_store_b128(v, r, off, 0, kStorePolicy);
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// Two fp32 -> packed bf16 pair, round to nearest even (the hardware convert).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    bf16x2_t v;
    v.x = static_cast<__bf16>(lo);
    v.y = static_cast<__bf16>(hi);
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ void unpack8(const u32x4 &v, float (&f)[8])
{
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x);
    f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z);
    f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}

__device__ __forceinline__ void add8(const u32x4 &v, float (&f)[8])
{
    f[0] += bf16_lo(v.x); f[1] += bf16_hi(v.x);
    f[2] += bf16_lo(v.y); f[3] += bf16_hi(v.y);
    f[4] += bf16_lo(v.z); f[5] += bf16_hi(v.z);
    f[6] += bf16_lo(v.w); f[7] += bf16_hi(v.w);
}

__device__ __forceinline__ u32x4 pack8(const float (&f)[8])
{
    u32x4 v;
    v.x = pack_bf16x2(f[0], f[1]);
    v.y = pack_bf16x2(f[2], f[3]);
    v.z = pack_bf16x2(f[4], f[5]);
    v.w = pack_bf16x2(f[6], f[7]);
    return v;
}

// v + (v moved across lanes by a DPP pattern). Used with patterns under which
// lanes pair up symmetrically, so both partners end with the same bits.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true);
    return v + __builtin_bit_cast(float, moved);
}
static constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
static constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
static constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7-i in each group of 8
static constexpr int kDppMirror = 0x140;      // lane i <-> 15-i in each group of 16

// Sum over aligned groups of 2^log2n lanes (log2n <= 6); every lane of a group
// ends with the same bits. After the first two steps each quad is uniform, so
// the mirrors act as "xor 4" and "xor 8".
__device__ __forceinline__ float group_sum(float v, int log2n)
{
    if (log2n >= 1) v = dpp_add<kDppXor1>(v);
    if (log2n >= 2) v = dpp_add<kDppXor2>(v);
    if (log2n >= 3) v = dpp_add<kDppHalfMirror>(v);
    if (log2n >= 4) v = dpp_add<kDppMirror>(v);
    if (log2n >= 5) v += __shfl_xor(v, 16, 64);
    if (log2n >= 6) v += __shfl_xor(v, 32, 64);
    return v;
}

}  // namespace tw
