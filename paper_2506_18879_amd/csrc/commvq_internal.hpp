// Shared by the translation units of libcommvq: constants, the handle, vector types and wavefront helpers.
#pragma once
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <new>
#include <utility>
#include <vector>

#include "commvq.h"
#include "commvq_launch.hpp"

namespace {

constexpr int kD = 128;         // head_dim
constexpr int kJ = 64;          // 2-D sub-spaces = lanes of a wavefront
constexpr int kK = 256;         // codewords per codebook
constexpr int kLoBits = 6;      // relative position = hi * 64 + lo
constexpr int kLo = 1 << kLoBits;
constexpr int kScoreMaxTpt = 4;      // slice-streaming score tile: at most 4 x 1024 tokens
constexpr int kScoreMinWgs = 2048;   // row-gather score kernel: tiles are halved until this many workgroups exist
constexpr int kScoreThreads = 256;
constexpr int kBinsThreads = 1024;
constexpr int kOutThreads = 256;
constexpr int kMaxValueSplits = 256;  // value_splits never exceeds 256 / (batch * KV heads), at least 1
constexpr int kOutRows = 64;    // codebook rows per k_out workgroup
constexpr int kOutMfmaRows = 256;   // codebook rows per k_out_mfma workgroup (batched output stage)
constexpr int kOutMfmaMinRows = 16;  // batch * (query heads per KV head) from which the batched output kernel is used
constexpr int kProfRing = 64;
constexpr float kLog2e = 1.4426950408889634f;

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

struct commvq_handle {
    commvq_config cfg;
    int G;
    float scale;
    int n_hi;
    int device;      // device ordinal of the phase tables; -1 for a planner handle (no device resources)
    float2 *tbl_hi;  // [n_hi][64]  exp(i * theta_j * 64 * hi)
    float2 *tbl_lo;  // [64][64]    exp(i * theta_j * lo)
    void *static_scratch;  // this device's copy of the library's static scratch array (commvq_decode_attn_static)
    int prof_every, prof_calls;  // stage events on every prof_every-th call (0: never)
    int prof_head, prof_count;
    hipEvent_t prof_ev[kProfRing][4];
    bool prof_ev_made;
    // key codebooks that the caller has had re-laid once (commvq_pack_key_codebooks): source pointer -> packed copy
    std::vector<std::pair<const void *, const uint4 *>> packed_keys;
    // value codebooks re-laid once for the batched output kernel (commvq_pack_value_codebooks): source -> packed copy
    std::vector<std::pair<const void *, const uint4 *>> packed_vals;
};

namespace {

typedef unsigned uint2_t __attribute__((ext_vector_type(2)));
typedef unsigned uint4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x16_t __attribute__((ext_vector_type(16)));
typedef unsigned uint8v_t __attribute__((ext_vector_type(8)));

// ------------------------------------------------------------------ device helpers
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// Sum over the 64 lanes of a wavefront; every lane receives the total.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_mov<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_mov<0x141>(v);  // row_half_mirror
    v += dpp_mov<0x140>(v);  // row_mirror: every lane now holds its 16-lane row sum
    unsigned u = __builtin_bit_cast(unsigned, v);
    auto r16 = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    v = __builtin_bit_cast(float, (unsigned)r16[0]) + __builtin_bit_cast(float, (unsigned)r16[1]);
    u = __builtin_bit_cast(unsigned, v);
    auto r32 = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, (unsigned)r32[0]) + __builtin_bit_cast(float, (unsigned)r32[1]);
}

__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_mov<0xB1>(v));
    v = fmaxf(v, dpp_mov<0x4E>(v));
    v = fmaxf(v, dpp_mov<0x141>(v));
    v = fmaxf(v, dpp_mov<0x140>(v));
    unsigned u = __builtin_bit_cast(unsigned, v);
    auto r16 = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    v = fmaxf(__builtin_bit_cast(float, (unsigned)r16[0]), __builtin_bit_cast(float, (unsigned)r16[1]));
    u = __builtin_bit_cast(unsigned, v);
    auto r32 = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, (unsigned)r32[0]), __builtin_bit_cast(float, (unsigned)r32[1]));
}

// element i of a bf16 or fp32 array, widened exactly
template <bool BF16>
__device__ __forceinline__ float cb_elem(const void *cb, size_t i)
{
    if (BF16) return __builtin_bit_cast(float, (unsigned)static_cast<const uint16_t *>(cb)[i] << 16);
    return static_cast<const float *>(cb)[i];
}

// 16 bytes per lane from global memory straight into LDS (no register destination): lane l of the wavefront lands at
// LDS byte address lds_byte_addr_uniform + 16 l.  Issued from inline asm, so the compiler makes no later access wait
// for it: the kernel waits itself (s_waitcnt vmcnt(0)) before the data is used.
__device__ __forceinline__ void lds_dma16(const void *gptr, unsigned lds_byte_addr_uniform)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_byte_addr_uniform), "v"(gptr) : "memory");
}

__device__ __forceinline__ float bf16_lo(unsigned v) { return __builtin_bit_cast(float, v << 16); }
__device__ __forceinline__ float bf16_hi(unsigned v) { return __builtin_bit_cast(float, v & 0xffff0000u); }

// acc + low / high bf16 half of a packed pair, in one v_dot2c_f32_bf16 each: the other half
// is multiplied by zero, so this is an exact fp32 add of the widened value.  The selector
// (1.0 in one half, 0 in the other) is passed through an opaque register so that it is never
// encoded as an inline constant, whose meaning for packed bf16 operands is ambiguous.
__device__ __forceinline__ unsigned opaque_sgpr(unsigned v)
{
    asm volatile("" : "+s"(v));
    return v;
}
__device__ __forceinline__ float add_bf16_sel(unsigned v, unsigned sel, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, v), __builtin_bit_cast(bf16x2_t, sel), acc, false);
}

}  // namespace
