// Pieces shared by the kernels that take their weights straight from memory in matrix-core operand
// order (conv_bneck.hip, conv_pw.hip): fragment reads with hand-placed waits, the operand loads,
// accumulator set-up and packing.
//
// Operand order of a weight matrix [rows][K] (K = taps x channels): blocks of 32 rows, steps of 16
// columns, [block][step][lane][8 bf16]; lane (r, h) holds row 32 block + r', columns 16 step + 8 h .. + 7,
// where r' is r with bits 2 and 3 swapped.  With the rows in that order a lane of a 32x32 result
// block holds, in register v, channel 16(v/8) + 8(lane/32) + v%8 of its position: two runs of 8.
#pragma once
#include "conv_common.h"

#include <type_traits>
#include <utility>

namespace ens {

typedef __attribute__((address_space(3))) void* lds_ptr_t;

template <int OFFSET>
__device__ __forceinline__ bf16x8 bn_lds_read(uint32_t addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
    return v;
}
// keeps the matrix-core instructions that use v behind the wait that precedes this statement
__device__ __forceinline__ void bn_tie(bf16x8& v) { asm volatile("" : "+v"(v)); }

template <class F, int... T>
__device__ __forceinline__ void bn_static_for(F&& f, std::integer_sequence<int, T...>) {
    (f(std::integral_constant<int, T>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void bn_unroll(F&& f) { bn_static_for(f, std::make_integer_sequence<int, N>{}); }

__device__ __forceinline__ void bn_zero(f32x16& acc) {
#pragma unroll
    for (int e = 0; e < 16; e++) acc[e] = 0.f;
}

// Scale and bias of a lane's two runs of 8 channels: sb points at the lane's first channel in a table
// (LDS) that holds the bias of the tile's channels and, `stride` floats further on, their scale.
// Registers 8k .. 8k+7 of a result block are the channels sb[16k .. 16k+7].
__device__ __forceinline__ void bn_affine8(float* v, const f32x16& acc, int k, const float* sb, int stride) {
    const f32x4 b0 = *(const f32x4*)(sb + 16 * k), b1 = *(const f32x4*)(sb + 16 * k + 4);
    const f32x4 s0 = *(const f32x4*)(sb + stride + 16 * k), s1 = *(const f32x4*)(sb + stride + 16 * k + 4);
#pragma unroll
    for (int e = 0; e < 4; e++) {
        v[e] = fmaf(acc[8 * k + e], s0[e], b0[e]);
        v[4 + e] = fmaf(acc[8 * k + 4 + e], s1[e], b1[e]);
    }
}

// registers 8k .. 8k+7 of a result block, scaled and biased per channel, with the activation, as 8 bf16
__device__ __forceinline__ u32x4 bn_pack(const f32x16& acc, int k, int act, const float* sb, int stride) {
    float v[8];
    bn_affine8(v, acc, k, sb, stride);
    apply_act_n<8>(v, act);
    return u32x4{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
}

// registers 8k .. 8k+7 of a result block, scaled and biased per channel, plus 8 bf16 of residual,
// activation applied, as 8 bf16
template <bool RES>
__device__ __forceinline__ u32x4 bn_pack_res(const f32x16& acc, int k, const u32x4& res, int act, const float* sb, int stride) {
    float v[8];
    bn_affine8(v, acc, k, sb, stride);
    if constexpr (RES) {
        const uint32_t rr[4] = {res.x, res.y, res.z, res.w};
#pragma unroll
        for (int q = 0; q < 4; q++) {
            v[2 * q] += bf16_to_f32((uint16_t)(rr[q] & 0xFFFF));
            v[2 * q + 1] += bf16_to_f32((uint16_t)(rr[q] >> 16));
        }
    }
    uint32_t o[4];
    if (act == ACT_RELU) {
#pragma unroll
        for (int q = 0; q < 4; q++) {                            // relu on the rounded pair: a negative bf16 is a negative 16-bit integer
            typedef short s16x2 __attribute__((ext_vector_type(2)));
            const s16x2 z = {0, 0};
            o[q] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, pack_bf16x2(v[2 * q], v[2 * q + 1])), z));
        }
    } else {
        apply_act_n<8>(v, act);
#pragma unroll
        for (int q = 0; q < 4; q++) o[q] = pack_bf16x2(v[2 * q], v[2 * q + 1]);
    }
    return u32x4{o[0], o[1], o[2], o[3]};
}

// One operand fragment of the packed weights: 16 bytes per lane, 1 KB in a row per wavefront.
__device__ __forceinline__ bf16x8 bn_wload(const __amdgpu_buffer_rsrc_t& r, unsigned vo, int so) {
    return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(r, vo, so, 0));
}

template <int N>
__device__ __forceinline__ void bn_wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

}  // namespace ens
