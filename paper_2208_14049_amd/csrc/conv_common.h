// Pieces shared by the convolution kernels: bf16 conversion, activations, the workgroup-to-tile
// mapping.
#pragma once
#include "kernels.h"

namespace ens {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float bf16_to_f32(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
    u += 0x7FFFu + ((u >> 16) & 1u);                                              // nearest even
    return (uint16_t)(u >> 16);
}
// Two floats to a packed pair of bf16 (round to nearest even) with the hardware conversion.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ float apply_act(float v, int act) {
    if (act == ACT_RELU) return fmaxf(v, 0.f);
    if (act == ACT_SILU) return v / (1.f + __expf(-v));
    return v;
}

// Bytes per lane of an asynchronous global-to-LDS load.  The 16-byte form exists on gfx950 only and
// the compiler checks the size against the target of the pass it is in: the host pass, which only
// needs the kernels' signatures, would silently drop a kernel template that names it.
#if defined(__HIP_DEVICE_COMPILE__)
constexpr int LDS_LOAD_BYTES = 16;
#else
constexpr int LDS_LOAD_BYTES = 4;
#endif

constexpr int BK = 64;          // K elements per LDS tile: one 128-byte row, 8 chunks of 16 bytes

// Workgroup id -> (pixel tile, channel tile).  Consecutive workgroup ids go to different XCDs
// (8 of them, each with its own L2), so ids are first regrouped per XCD and the channel tiles of
// one pixel tile are made neighbours there: they read the same activations from one L2.
__device__ __forceinline__ void tile_of_block(int n_ptiles, int n_ctiles, int* ptile, int* ctile) {
    const int total = n_ptiles * n_ctiles;
    int v = blockIdx.x;
    const int per = total / 8;
    if (v < per * 8) v = (v % 8) * per + v / 8;
    *ctile = v % n_ctiles;
    *ptile = v / n_ctiles;
}

// Register-staged variant (pre-activated inputs); defined in conv_regstage.hip.
hipError_t launch_conv_regstage(const ConvArgs& a, const ConvArgs* argv, int G, int nb, int P, hipStream_t s);
const char* conv_regstage_name(const ConvArgs& a, int P);

// Second pass of a convolution whose K range was split: sums the `splits` fp32 slices of P x cout
// partial sums in the workspace and applies bias, residual and activation; defined in conv_mfma.hip.
hipError_t launch_conv_splitk_epilogue(const ConvArgs& a, const ConvArgs* argv, int G, int nb, int P, int splits, hipStream_t s);

// 3x3 stride-1 kernel with the input window resident in LDS; defined in conv_halo.hip.
// conv_halo_pick returns the variant that runs the layer, or -1 when the generic kernel does.
int conv_halo_pick(const ConvArgs& a, int nb, int G);
const char* conv_halo_name(int variant);
hipError_t launch_conv_halo(const ConvArgs& a, const ConvArgs* argv, int G, int nb, int variant, hipStream_t s);

}  // namespace ens
