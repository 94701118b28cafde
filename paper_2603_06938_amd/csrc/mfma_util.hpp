// Device helpers shared by the bf16 MFMA kernels (v_mfma_f32_32x32x16_bf16).  Lane l of a wave holds
//   A[row = l%32][k = 8*(l/32) + 0..7],  B[k = 8*(l/32) + 0..7][col = l%32],
//   C[row = 8*(v/4) + 4*(l/32) + v%4][col = l%32] in accumulator register v.
// The k index of a contraction may be permuted freely as long as A and B use the same permutation.
#pragma once

#include "common.hpp"

namespace swimba {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int MP = 64;    // headdim
constexpr int MN = 128;   // state size
constexpr int MTHREADS = 256;

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2_t f = {lo, hi};
    bf16x2_t h = __builtin_convertvector(f, bf16x2_t);   // round to nearest even
    return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ f32x16_t mfma32(uint4 a, uint4 b, f32x16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// acc[0..7] += wgt * (8 bf16 values packed in u)
__device__ __forceinline__ void fma_bf16x8(float *acc, uint4 u, float wgt)
{
    acc[0] += wgt * bf_lo(u.x); acc[1] += wgt * bf_hi(u.x);
    acc[2] += wgt * bf_lo(u.y); acc[3] += wgt * bf_hi(u.y);
    acc[4] += wgt * bf_lo(u.z); acc[5] += wgt * bf_hi(u.z);
    acc[6] += wgt * bf_lo(u.w); acc[7] += wgt * bf_hi(u.w);
}
__device__ __forceinline__ void unpack8(float *a, uint4 u)
{
    a[0] = bf_lo(u.x); a[1] = bf_hi(u.x); a[2] = bf_lo(u.y); a[3] = bf_hi(u.y);
    a[4] = bf_lo(u.z); a[5] = bf_hi(u.z); a[6] = bf_lo(u.w); a[7] = bf_hi(u.w);
}
__device__ __forceinline__ uint4 pack8(const float *a)
{
    return make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(a[4], a[5]),
                      pack_bf16x2(a[6], a[7]));
}

// Token held at position `pos` of a chunk in the token-innermost operand layouts (mixed B with 8
// tokens innermost, the transposed x tiles in LDS): bits 2 and 3 of the position swapped.  A 32x32
// accumulator tile whose rows are tokens gives lane group kg the rows 8a + 4kg + b; read as the
// B operand of the next contraction, its k-step t covers tokens 16t + 8a + 4kg + b (a = 0,1), which
// are the 8 consecutive positions 16t + 8kg + 4a + b of this order.
__host__ __device__ __forceinline__ int t8_token(int pos) { return (pos & ~12) | ((pos & 4) << 1) | ((pos & 8) >> 1); }

// Workgroups are handed to the 8 XCDs round-robin by block id.  This maps a
// block id to a logical id such that each XCD works on one contiguous range of
// logical ids (neighbouring heads of one chunk share the group's tiles in that
// XCD's L2).  The grid is padded to a multiple of 8; ids >= total do nothing.
__device__ __forceinline__ int xcd_logical_id(int bid, int nblocks)
{
    const int per = nblocks >> 3;
    return (bid & 7) * per + (bid >> 3);
}
static inline int xcd_padded(int64_t total) { return (int)((total + 7) / 8 * 8); }

// 16-byte accesses that are not worth caching (read once / written once by this kernel)
typedef unsigned int __attribute__((ext_vector_type(4))) u32x4_t;
__device__ __forceinline__ uint4 load_nt(const uint16_t *p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_nt(uint16_t *p, uint4 v)
{
    const u32x4_t pv = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(pv, reinterpret_cast<u32x4_t *>(p));
}

__device__ __forceinline__ float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }

constexpr float LOG2E = 1.4426950408889634f;

// =========================================================================================
// cb tile of one wave: pair p = I(I+1)/2 + J, J <= I, of one (batch, chunk, group):
//   cb (B, nc, G, NP, 2, 64, 8) bf16: the accumulator registers v = 8t..8t+7 of lane l
//   of G^T[j][i] = Bmix_j . Cmix_i  (32 x 32 tile)
// Both operands are read as the register images mix_rows stored.
// =========================================================================================
__device__ __forceinline__ void cb_pair(const uint16_t *__restrict__ cmix, const uint16_t *__restrict__ bfrag,
                                        uint16_t *__restrict__ cb, int NT, int64_t bcg, int p, int lane)
{
    const int NP = NT * (NT + 1) / 2;
    int I = 0;
    while ((I + 1) * (I + 2) / 2 <= p) ++I;
    const int J = p - I * (I + 1) / 2;
    const uint16_t *cs = cmix + (((bcg * NT + I) * 8) * 64 + lane) * 8;
    const uint16_t *bs = bfrag + (((bcg * NT + J) * 8) * 64 + lane) * 8;
    uint4 cf[8], bf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        cf[ks] = *reinterpret_cast<const uint4 *>(cs + ks * 64 * 8);
        bf[ks] = *reinterpret_cast<const uint4 *>(bs + ks * 64 * 8);
    }
    f32x16_t acc = {0};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) acc = mfma32(bf[ks], cf[ks], acc);
    float m[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) m[v] = acc[v];
    uint16_t *dst = cb + ((bcg * NP + p) * 2 * 64 + lane) * 8;
    *reinterpret_cast<uint4 *>(dst) = pack8(m);
    *reinterpret_cast<uint4 *>(dst + 64 * 8) = pack8(m + 8);
}

}  // namespace swimba
