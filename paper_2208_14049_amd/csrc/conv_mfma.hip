// Implicit-GEMM convolution on the CDNA4 matrix cores (gfx950), bf16 in, fp32 accumulate.
//
// GEMM view of a convolution over NHWC activations:
//   rows    P = nb*Ho*Wo output pixels
//   columns cout output channels
//   depth   K = kh*kw*cin, input channel fastest, so 8 consecutive k are 16 contiguous bytes
//           both in the activation tensor (one pixel, one tap) and in the [cout][K] weights.
// A workgroup of 4 wavefronts computes a BP x BC tile of the output; the K loop walks tiles of
// 32 through double-buffered LDS.  The weights are the A operand of v_mfma_f32_32x32x16_bf16 and
// the pixels the B operand, so a lane of the accumulator holds one pixel and runs of four
// consecutive output channels: the epilogue (bias, residual, activation) packs each run into one
// 8-byte store.
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
__device__ __forceinline__ float apply_act(float v, int act) {
    if (act == ACT_RELU) return fmaxf(v, 0.f);
    if (act == ACT_SILU) return v / (1.f + __expf(-v));
    return v;
}

constexpr int BK = 32;          // K elements per LDS tile
constexpr int LDK = BK + 8;     // padded LDS row (elements): rows start 80 bytes apart

template <int BP, int BC, int WP, int WC, bool PRE>
__global__ __launch_bounds__(256) void conv_igemm_bf16(const ConvArgs a, const int P, const int K) {
    static_assert(WP * WC == 4, "four wavefronts per workgroup");
    constexpr int WTP = BP / WP, WTC = BC / WC;      // wave tile
    constexpr int TP = WTP / 32, TC = WTC / 32;      // 32x32 blocks per wave
    static_assert(TP >= 1 && TC >= 1, "wave tile must hold a 32x32 block");
    constexpr int NPL = (BP + 63) / 64, NCL = (BC + 63) / 64;   // 16-byte chunks per thread and tile

    __shared__ __attribute__((aligned(16))) uint16_t Xs[2][BP][LDK];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[2][BC][LDK];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wp0 = (wave % WP) * WTP, wc0 = (wave / WP) * WTC;
    const int n_ptiles = (P + BP - 1) / BP;
    const int ptile = blockIdx.x % n_ptiles, ctile = blockIdx.x / n_ptiles;
    const int p0 = ptile * BP, c0 = ctile * BC;

    const uint16_t* __restrict__ xg = (const uint16_t*)a.x.p;
    const uint16_t* __restrict__ wg = (const uint16_t*)a.w;

    // ---- per-thread load coordinates: chunk column q (8 elements), rows r0 + 64*i
    const int q = t & 3, r0 = t >> 2;
    const int cpt = a.cin >> 3;                 // 16-byte chunks per filter tap
    const int ntaps = a.kh * a.kw;
    int hi0[NPL], wi0[NPL];
    const uint16_t* xb[NPL];
#pragma unroll
    for (int i = 0; i < NPL; i++) {
        const int r = r0 + 64 * i;
        const int p = p0 + r;
        if (r < BP && p < P) {
            const int n = p / (a.Ho * a.Wo);
            const int rem = p - n * (a.Ho * a.Wo);
            const int ho = rem / a.Wo, wo = rem - ho * a.Wo;
            hi0[i] = ho * a.sh - a.pt;
            wi0[i] = wo * a.sw - a.pl;
            xb[i] = xg + (size_t)n * a.H * a.W * a.x.stride + a.x.c0;
        } else {
            hi0[i] = -(1 << 28);                // never in bounds
            wi0[i] = 0;
            xb[i] = xg;
        }
    }
    const uint16_t* wb[NCL];
    bool wvalid[NCL];
#pragma unroll
    for (int i = 0; i < NCL; i++) {
        const int r = r0 + 64 * i;
        wvalid[i] = (r < BC) && (c0 + r < a.cout);
        wb[i] = wg + (size_t)(wvalid[i] ? (c0 + r) : 0) * K;
    }

    // position of this thread's chunk in the K walk
    int kc = q;                                  // chunk index along K
    int tap = kc / cpt, cq = kc - tap * cpt;
    int khi = tap / a.kw, kwi = tap - khi * a.kw;

    uint4 xr[NPL], wr[NCL];
    auto load_tile = [&]() {
#pragma unroll
        for (int i = 0; i < NPL; i++) {
            uint4 v = make_uint4(0, 0, 0, 0);
            const int hi = hi0[i] + khi, wi = wi0[i] + kwi;
            if (tap < ntaps && hi >= 0 && hi < a.H && wi >= 0 && wi < a.W) {
                v = *(const uint4*)(xb[i] + ((size_t)hi * a.W + wi) * a.x.stride + cq * 8);
                if (PRE) {
                    const float4 s0 = *(const float4*)(a.pre_scale + cq * 8);
                    const float4 s1 = *(const float4*)(a.pre_scale + cq * 8 + 4);
                    const float4 h0 = *(const float4*)(a.pre_shift + cq * 8);
                    const float4 h1 = *(const float4*)(a.pre_shift + cq * 8 + 4);
                    const float sc[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
                    const float sf[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
                    uint32_t in[4] = {v.x, v.y, v.z, v.w}, out[4];
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        float lo = bf16_to_f32((uint16_t)(in[e] & 0xFFFF));
                        float hi_ = bf16_to_f32((uint16_t)(in[e] >> 16));
                        lo = fmaxf(lo * sc[2 * e] + sf[2 * e], 0.f);
                        hi_ = fmaxf(hi_ * sc[2 * e + 1] + sf[2 * e + 1], 0.f);
                        out[e] = (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi_) << 16);
                    }
                    v = make_uint4(out[0], out[1], out[2], out[3]);
                }
            }
            xr[i] = v;
        }
#pragma unroll
        for (int i = 0; i < NCL; i++) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (wvalid[i] && kc * 8 < K) v = *(const uint4*)(wb[i] + (size_t)kc * 8);
            wr[i] = v;
        }
    };
    auto advance = [&]() {
        kc += 4;
        cq += 4;
        while (cq >= cpt) {
            cq -= cpt;
            tap++;
            if (++kwi == a.kw) { kwi = 0; khi++; }
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NPL; i++) {
            const int r = r0 + 64 * i;
            if (r < BP) *(uint4*)&Xs[buf][r][q * 8] = xr[i];
        }
#pragma unroll
        for (int i = 0; i < NCL; i++) {
            const int r = r0 + 64 * i;
            if (r < BC) *(uint4*)&Ws[buf][r][q * 8] = wr[i];
        }
    };

    f32x16 acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int j = 0; j < TP; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

    const int nk = (K + BK - 1) / BK;
    load_tile();
    store_tile(0);
    __syncthreads();
    const int lrow = lane & 31, lk = (lane >> 5) * 8;
    for (int kt = 0; kt < nk; kt++) {
        const int buf = kt & 1;
        if (kt + 1 < nk) {
            advance();
            load_tile();
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ks++) {
            bf16x8 wf[TC], xf[TP];
#pragma unroll
            for (int i = 0; i < TC; i++) wf[i] = *(const bf16x8*)&Ws[buf][wc0 + i * 32 + lrow][ks * 16 + lk];
#pragma unroll
            for (int j = 0; j < TP; j++) xf[j] = *(const bf16x8*)&Xs[buf][wp0 + j * 32 + lrow][ks * 16 + lk];
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int j = 0; j < TP; j++)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            store_tile(buf ^ 1);
            __syncthreads();
        }
    }

    // ---- epilogue: accumulator lane = pixel (lane & 31), register v = channel
    //      8*(v/4) + 4*(lane/32) + v%4 of the 32x32 block
    uint16_t* __restrict__ yg = (uint16_t*)a.y.p;
    const uint16_t* __restrict__ rg = (const uint16_t*)a.res.p;
#pragma unroll
    for (int j = 0; j < TP; j++) {
        const int p = p0 + wp0 + j * 32 + lrow;
        if (p >= P) continue;
#pragma unroll
        for (int i = 0; i < TC; i++) {
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const int co = c0 + wc0 + i * 32 + g * 8 + (lane >> 5) * 4;
                if (co >= a.cout) continue;
                const float4 b = *(const float4*)(a.bias + co);
                float v0 = acc[i][j][g * 4 + 0] + b.x, v1 = acc[i][j][g * 4 + 1] + b.y;
                float v2 = acc[i][j][g * 4 + 2] + b.z, v3 = acc[i][j][g * 4 + 3] + b.w;
                if (rg) {
                    const uint2 r = *(const uint2*)(rg + (size_t)p * a.res.stride + a.res.c0 + co);
                    v0 += bf16_to_f32((uint16_t)(r.x & 0xFFFF));
                    v1 += bf16_to_f32((uint16_t)(r.x >> 16));
                    v2 += bf16_to_f32((uint16_t)(r.y & 0xFFFF));
                    v3 += bf16_to_f32((uint16_t)(r.y >> 16));
                }
                v0 = apply_act(v0, a.act); v1 = apply_act(v1, a.act);
                v2 = apply_act(v2, a.act); v3 = apply_act(v3, a.act);
                uint2 o;
                o.x = (uint32_t)f32_to_bf16(v0) | ((uint32_t)f32_to_bf16(v1) << 16);
                o.y = (uint32_t)f32_to_bf16(v2) | ((uint32_t)f32_to_bf16(v3) << 16);
                *(uint2*)(yg + (size_t)p * a.y.stride + a.y.c0 + co) = o;
            }
        }
    }
}

double conv_flops(const ConvArgs& a) {
    return 2.0 * (double)a.nb * a.Ho * a.Wo * a.cout * a.kh * a.kw * a.cin;
}

template <int BP, int BC, int WP, int WC>
static hipError_t launch_variant(const ConvArgs& a, int P, int K, hipStream_t s) {
    const int grid = ((P + BP - 1) / BP) * ((a.cout + BC - 1) / BC);
    if (a.pre_scale)
        hipLaunchKernelGGL((conv_igemm_bf16<BP, BC, WP, WC, true>), dim3(grid), dim3(256), 0, s, a, P, K);
    else
        hipLaunchKernelGGL((conv_igemm_bf16<BP, BC, WP, WC, false>), dim3(grid), dim3(256), 0, s, a, P, K);
    return hipGetLastError();
}

// Tile choice: narrow layers take a 32- or 64-channel tile so no matrix-core work is spent on
// padding channels; everything else takes the square 128 x 128 tile.
static int pick_variant(const ConvArgs& a) {
    if (a.cout <= 32) return 0;
    if (a.cout <= 64 || (a.cout % 128 != 0 && a.cout % 128 <= 64)) return 1;
    return 2;
}

const char* conv_bf16_variant_name(const ConvArgs& a) {
    static const char* names[3] = {"conv_igemm_bf16<256,32>", "conv_igemm_bf16<128,64>", "conv_igemm_bf16<128,128>"};
    return names[pick_variant(a)];
}

hipError_t launch_conv_bf16(const ConvArgs& a, hipStream_t s) {
    // shapes the kernel assumes: 16-byte chunks along the channels, 8-byte runs on the way out
    if (a.cin % 8 || a.x.stride % 8 || a.x.c0 % 8) return hipErrorInvalidValue;
    if (a.cout % 8 || a.y.stride % 4 || a.y.c0 % 4) return hipErrorInvalidValue;
    if (a.res.p && (a.res.stride % 4 || a.res.c0 % 4)) return hipErrorInvalidValue;
    if (a.nb <= 0 || a.cin <= 0 || a.cout <= 0 || !a.bias) return hipErrorInvalidValue;
    if ((a.pre_scale == nullptr) != (a.pre_shift == nullptr)) return hipErrorInvalidValue;
    const long long P64 = (long long)a.nb * a.Ho * a.Wo;
    const long long K64 = (long long)a.kh * a.kw * a.cin;
    if (P64 <= 0 || P64 >= (1LL << 31) || K64 >= (1LL << 31)) return hipErrorInvalidValue;
    const int P = (int)P64, K = (int)K64;
    switch (pick_variant(a)) {
        case 0: return launch_variant<256, 32, 4, 1>(a, P, K, s);
        case 1: return launch_variant<128, 64, 2, 2>(a, P, K, s);
        default: return launch_variant<128, 128, 2, 2>(a, P, K, s);
    }
}

}  // namespace ens
