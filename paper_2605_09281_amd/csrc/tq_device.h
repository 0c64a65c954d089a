// Device helpers shared by the MFMA translation units (fragment types, bf16/fp16 conversions, the
// nibble unpack).  Internal to libtileq.
#pragma once

#include "tq_common.h"

namespace tqdev {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct MGeom {
    int32_t ne, H, F, g, r, r16, k, S, a_tot;
    uint32_t unpack_mask, unpack_magic;   // 0x000F000F, 0x43004300 (see unpack_word)
    size_t expert_stride;
    TqFactorMap fm;
    const uint8_t* zc_ws;      // zero-point coefficient fragments outside the blob (dense codes), or null
    size_t zc_stride, zc_d_off;
};

// base of the zero-point coefficient fragments of expert e in section sec_id (0 GU, 1 D)
__device__ inline const uint8_t* tq_zc_base(const MGeom& G, const uint8_t* blob, const TqSection& sec, int sec_id, int e)
{
    if (G.zc_ws) return G.zc_ws + (size_t)e * G.zc_stride + (sec_id ? G.zc_d_off : 0);
    return blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride + sec.zc;
}

union Frag {
    bf16x8 v;
    uint32_t u[4];
    u32x4 q;
};

// fp32 -> bf16, round to nearest even.  Written as vector conversions so that the compiler selects the hardware
// conversion of this target (one instruction per pair) instead of an integer rounding sequence.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pack_bf2(float a, float b)
{
    const f32x2_t v = {a, b};
    const bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
    uint32_t u;
    __builtin_memcpy(&u, &r, 4);
    return u;
}
__device__ inline uint32_t f2bf_bits(float f) { return pack_bf2(f, 0.f) & 0xFFFFu; }
// two fp16 values in one word -> two bf16 values in one word
__device__ inline uint32_t half2_to_bf2(uint32_t w)
{
    f16x2_t h;
    __builtin_memcpy(&h, &w, 4);
    const f32x2_t f = __builtin_convertvector(h, f32x2_t);
    const bf16x2_t r = __builtin_convertvector(f, bf16x2_t);
    uint32_t u;
    __builtin_memcpy(&u, &r, 4);
    return u;
}
__device__ inline float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// 8 codes of one packed word -> bf16 values 128 + q, in contraction order.  mask = 0x000F000F and
// magic = 0x43004300 arrive as kernel arguments rather than literals: the three-operand and-or encoding
// takes no literal on this target, and with register operands the compiler selects it (7 VALU
// instructions per word instead of 11).
__device__ inline bf16x8 unpack_word(uint32_t w, uint32_t mask, uint32_t magic)
{
    Frag f;
    f.u[0] = (w & mask) | magic;
    f.u[1] = ((w >> 4) & mask) | magic;
    f.u[2] = ((w >> 8) & mask) | magic;
    f.u[3] = ((w >> 12) & mask) | magic;
    return f.v;
}

// Dense 2- or 3-bit codes (CW = bits = words per lane and 64-wide chunk): the four bf16 pairs of k-step `w` (0..3) of
// the chunk held in d[0..CW-1].  Slot P = 4 w + j holds two codes 16 bit positions apart; mask = 0x00030003 or
// 0x00070007.  `w` is a constant at every call site (unrolled loops), so the word and shift of each slot fold.
template <int CW>
__device__ inline bf16x8 unpack_dense(const uint32_t* d, int w, uint32_t mask, uint32_t magic)
{
    Frag f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int P = 4 * w + j;
        if (CW == 2) {
            const int p = 2 * (P % 8);
            f.u[j] = ((p ? d[P / 8] >> p : d[P / 8]) & mask) | magic;
        } else if (P < 15) {
            const int p = 3 * (P % 5);
            f.u[j] = ((p ? d[P / 5] >> p : d[P / 5]) & mask) | magic;
        } else {        // the last slot of a 3-bit chunk is spread over the spare bits 15 and 31 of the three words
            f.u[j] = ((d[0] >> 15) & 0x00010001u) | ((d[1 % CW] >> 14) & 0x00020002u) | ((d[2 % CW] >> 13) & 0x00040004u) | magic;
        }
    }
    return f.v;
}

__device__ inline bf16x8 half8_to_bf8(u32x4 q)
{
    Frag f;
#pragma unroll
    for (int j = 0; j < 4; ++j) f.u[j] = half2_to_bf2(q[j]);
    return f.v;
}

// eight fp8 E4M3 values (two dwords) -> the bf16 operand of one MFMA step; exact: E4M3 has three mantissa bits
__device__ inline bf16x8 fp8x8_to_bf8(uint32_t d0, uint32_t d1)
{
    Frag f;
    const uint32_t d[2] = {d0, d1};
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8(d[q], false);
        const auto hi = __builtin_amdgcn_cvt_pk_f32_fp8(d[q], true);
        f.u[2 * q] = (__float_as_uint(lo[0]) >> 16) | (__float_as_uint(lo[1]) & 0xFFFF0000u);
        f.u[2 * q + 1] = (__float_as_uint(hi[0]) >> 16) | (__float_as_uint(hi[1]) & 0xFFFF0000u);
    }
    return f.v;
}

// fp8 factor fragments keep the fp16 layouts with 1-byte elements: fragment f of a part sits at byte 512 f, lane l's
// eight codes at 8 l.  Lanes 2j and 2j + 1 share a 16-byte word: every lane loads that word (no 8-byte load under a
// condition next to the streams) and keeps its half.
__device__ inline bf16x8 fp8_frag_to_bf8(const u32x4& word, int lane)
{
    const uint32_t d0 = (lane & 1) ? word[2] : word[0];
    const uint32_t d1 = (lane & 1) ? word[3] : word[1];
    return fp8x8_to_bf8(d0, d1);
}

__device__ inline uint32_t word_of(const u32x4& q, int w) { return q[w]; }

// silu(g) * u with the hardware exp2 and reciprocal (about 1 ulp each; the result is rounded to bf16 anyway):
// a plain division expands to a ten-instruction sequence per element
__device__ inline float silu_mul(float g, float u)
{
    const float e = __builtin_amdgcn_exp2f(g * -1.4426950408889634f);
    return g * __builtin_amdgcn_rcpf(1.0f + e) * u;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding global
// load (one counter covers loads and stores on this target), which would drain the register prefetch of the
// packed codes at every barrier.  All cross-thread traffic of the kernels that use this goes through LDS.
__device__ inline void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

}  // namespace tqdev

// persistent-workgroup prefill kernels: one projection stage (0: gate/up + SwiGLU -> h, 1: down -> bf16 rows)
bool tqi_prefill_supported(const TqLayout& L, const TqWorkspace& W, int32_t T);
tq_status tqi_forward_prefill_stage(int stage, const TqLayout& L, const TqWorkspace& W, const tqdev::MGeom& G,
                                    const uint8_t* blob, const uint16_t* xin, const uint16_t* xaug,
                                    const int32_t* row_token, const int32_t* tile_e, const int32_t* tile_row0,
                                    const int32_t* offsets, const int32_t* ctrl, int ctrl_idx, void* out,
                                    hipStream_t st);
