// Register-staged implicit-GEMM convolution (bf16, fp32 accumulate) for layers whose input
// needs arithmetic on the way in: the pre-activated convolutions of dense blocks apply
// relu(x * scale + shift) per input channel to every in-bounds value before it reaches the matrix
// cores, which the asynchronous global-to-LDS path of the main kernel cannot do.  Same tiling and
// LDS layout as the main kernel; global loads go through registers, one K tile ahead.
#include "conv_common.h"

namespace ens {

template <int BP, int BC, int WP, int WC, bool PRE>
__global__ __launch_bounds__(256) void conv_regstage_bf16(const ConvArgs* __restrict__ argv, const int nb_) {
    ConvArgs a = argv[blockIdx.z];
    a.nb = nb_;
    const int P = nb_ * a.Ho * a.Wo, K = a.kh * a.kw * a.cin;
    static_assert(WP * WC == 4, "four wavefronts per workgroup");
    constexpr int WTP = BP / WP, WTC = BC / WC;      // wave tile
    constexpr int TP = WTP / 32, TC = WTC / 32;      // 32x32 blocks per wave
    static_assert(TP >= 1 && TC >= 1, "wave tile must hold a 32x32 block");
    static_assert(BP % 32 == 0 && BC % 32 == 0, "tiles are multiples of 32");
    constexpr int NPL = BP / 32, NCL = BC / 32;      // 16-byte chunks per thread and tile

    __shared__ __attribute__((aligned(128))) uint16_t Xs[2][BP][BK];
    __shared__ __attribute__((aligned(128))) uint16_t Ws[2][BC][BK];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wp0 = (wave % WP) * WTP, wc0 = (wave / WP) * WTC;
    const int n_ptiles = (P + BP - 1) / BP, n_ctiles = (a.cout + BC - 1) / BC;
    int ptile, ctile;
    tile_of_block(n_ptiles, n_ctiles, &ptile, &ctile);
    const int p0 = ptile * BP, c0 = ctile * BC;

    const uint16_t* __restrict__ xg = (const uint16_t*)a.x.p;
    const uint16_t* __restrict__ wg = (const uint16_t*)a.w;

    const int nk = (K + BK - 1) / BK;
    const int kt0 = 0;

    // ---- per-thread load coordinates: chunk q of rows r0 + 32*i
    const int q = t & 7, r0 = t >> 3;
    const int slot = (q ^ ((r0 >> 1) & 7)) * 8;                  // swizzled element offset in the LDS row
    const int cpt = a.cin >> 3;                                  // 16-byte chunks per filter tap
    const int ntaps = a.kh * a.kw;
    int hi0[NPL], wi0[NPL];
    const uint16_t* xb[NPL];
#pragma unroll
    for (int i = 0; i < NPL; i++) {
        const int p = p0 + r0 + 32 * i;
        if (p < P) {
            const int n = p / (a.Ho * a.Wo);
            const int rem = p - n * (a.Ho * a.Wo);
            const int ho = rem / a.Wo, wo = rem - ho * a.Wo;
            hi0[i] = ho * a.sh - a.pt;
            wi0[i] = wo * a.sw - a.pl;
            xb[i] = xg + (size_t)n * a.H * a.W * a.x.stride + a.x.c0;
        } else {
            hi0[i] = -(1 << 28);                                 // never in bounds
            wi0[i] = 0;
            xb[i] = xg;
        }
    }
    const uint16_t* wb[NCL];
    bool wvalid[NCL];
#pragma unroll
    for (int i = 0; i < NCL; i++) {
        const int r = r0 + 32 * i;
        wvalid[i] = c0 + r < a.cout;
        wb[i] = wg + (size_t)(wvalid[i] ? (c0 + r) : 0) * K;
    }

    // position of this thread's chunk in the K walk: chunk kc -> (tap, channel chunk).  The
    // quotients are tiny (at most 49 taps), so a float multiply with a half-step guard is exact.
    int kc = kt0 * 8 + q;
    const float inv_cpt = 1.0f / (float)cpt, inv_kw = 1.0f / (float)a.kw;
    int tap, cq, khi, kwi;
    auto locate = [&]() {
        tap = (int)(((float)kc + 0.5f) * inv_cpt);
        cq = kc - tap * cpt;
        khi = (int)(((float)tap + 0.5f) * inv_kw);
        kwi = tap - khi * a.kw;
    };
    locate();

    uint4 xr[NPL], wr[NCL];
    // Loads are unconditional: an out-of-image tap or an out-of-range row reads the first bytes of
    // the tensor instead and is replaced by zeros afterwards, so that the wavefront issues all its
    // loads back to back.
    auto load_tile = [&]() {
        const bool tap_ok = tap < ntaps;
#pragma unroll
        for (int i = 0; i < NPL; i++) {
            const int hi = hi0[i] + khi, wi = wi0[i] + kwi;
            const bool ok = tap_ok && hi >= 0 && hi < a.H && wi >= 0 && wi < a.W;
            const uint16_t* src = ok ? xb[i] + ((size_t)hi * a.W + wi) * a.x.stride + cq * 8 : xg;
            uint4 v = *(const uint4*)src;
            if (PRE) {
                const int cc = ok ? cq * 8 : 0;
                const float4 s0 = *(const float4*)(a.pre_scale + cc);
                const float4 s1 = *(const float4*)(a.pre_scale + cc + 4);
                const float4 h0 = *(const float4*)(a.pre_shift + cc);
                const float4 h1 = *(const float4*)(a.pre_shift + cc + 4);
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
            xr[i] = ok ? v : make_uint4(0, 0, 0, 0);
        }
        const bool k_ok = kc * 8 < K;
#pragma unroll
        for (int i = 0; i < NCL; i++) {
            const bool ok = wvalid[i] && k_ok;
            const uint4 v = *(const uint4*)(ok ? wb[i] + (size_t)kc * 8 : wg);
            wr[i] = ok ? v : make_uint4(0, 0, 0, 0);
        }
    };
    auto advance = [&]() {
        kc += 8;
        locate();
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NPL; i++) *(uint4*)&Xs[buf][r0 + 32 * i][slot] = xr[i];
#pragma unroll
        for (int i = 0; i < NCL; i++) *(uint4*)&Ws[buf][r0 + 32 * i][slot] = wr[i];
    };

    f32x16 acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int j = 0; j < TP; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

    if (nk > 0) {
        load_tile();
        store_tile(0);
    }
    __syncthreads();
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int lsw = (lrow >> 1) & 7;           // every fragment row of this lane is lrow + 32*j: same swizzle key
    for (int kt = 0; kt < nk; kt++) {
        const int buf = kt & 1;
        if (kt + 1 < nk) {
            advance();
            load_tile();
        }
        // all fragments of the tile first (one burst of LDS reads), then the matrix-core work
        bf16x8 wf[BK / 16][TC], xf[BK / 16][TP];
#pragma unroll
        for (int ks = 0; ks < BK / 16; ks++) {
            const int off = (((ks * 2 + lhalf) ^ lsw)) * 8;
#pragma unroll
            for (int i = 0; i < TC; i++) wf[ks][i] = *(const bf16x8*)&Ws[buf][wc0 + i * 32 + lrow][off];
#pragma unroll
            for (int j = 0; j < TP; j++) xf[ks][j] = *(const bf16x8*)&Xs[buf][wp0 + j * 32 + lrow][off];
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ks++)
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int j = 0; j < TP; j++)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ks][i], xf[ks][j], acc[i][j], 0, 0, 0);
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
                const int co = c0 + wc0 + i * 32 + g * 8 + lhalf * 4;
                if (co >= a.cout) continue;
                float v0 = acc[i][j][g * 4 + 0], v1 = acc[i][j][g * 4 + 1];
                float v2 = acc[i][j][g * 4 + 2], v3 = acc[i][j][g * 4 + 3];
                const float4 b = *(const float4*)(a.bias + co), m = *(const float4*)(a.scale + co);
                v0 = fmaf(v0, m.x, b.x); v1 = fmaf(v1, m.y, b.y); v2 = fmaf(v2, m.z, b.z); v3 = fmaf(v3, m.w, b.w);
                if (rg) {
                    const uint2 r = *(const uint2*)(rg + (size_t)p * a.res.stride + a.res.c0 + co);
                    v0 += bf16_to_f32((uint16_t)(r.x & 0xFFFF));
                    v1 += bf16_to_f32((uint16_t)(r.x >> 16));
                    v2 += bf16_to_f32((uint16_t)(r.y & 0xFFFF));
                    v3 += bf16_to_f32((uint16_t)(r.y >> 16));
                }
                { float vv[4] = {v0, v1, v2, v3}; apply_act_n<4>(vv, a.act); v0 = vv[0]; v1 = vv[1]; v2 = vv[2]; v3 = vv[3]; }
                uint2 o;
                o.x = (uint32_t)f32_to_bf16(v0) | ((uint32_t)f32_to_bf16(v1) << 16);
                o.y = (uint32_t)f32_to_bf16(v2) | ((uint32_t)f32_to_bf16(v3) << 16);
                *(uint2*)(yg + (size_t)p * a.y.stride + a.y.c0 + co) = o;
            }
        }
    }
}


template <int BP, int BC, int WP, int WC>
static hipError_t launch_rs(const ConvArgs& a, const ConvArgs* argv, int G, int nb, int P, hipStream_t s) {
    const dim3 grid(((P + BP - 1) / BP) * ((a.cout + BC - 1) / BC), 1, G);
    if (a.pre_scale)
        ENS_LAUNCH((conv_regstage_bf16<BP, BC, WP, WC, true>), grid, dim3(256), 0, s, argv, nb);
    else
        ENS_LAUNCH((conv_regstage_bf16<BP, BC, WP, WC, false>), grid, dim3(256), 0, s, argv, nb);
    return hipGetLastError();
}

const char* conv_regstage_name(const ConvArgs& a, int P) {
    if (a.cout <= 32) return "conv_regstage_bf16<256,32>";
    if (((P + 127) / 128) * ((a.cout + 63) / 64) >= 512) return "conv_regstage_bf16<128,64>";
    return "conv_regstage_bf16<64,64>";
}

hipError_t launch_conv_regstage(const ConvArgs& a, const ConvArgs* argv, int G, int nb, int P, hipStream_t s) {
    if (a.cout <= 32) return launch_rs<256, 32, 4, 1>(a, argv, G, nb, P, s);
    if (((P + 127) / 128) * ((a.cout + 63) / 64) >= 512) return launch_rs<128, 64, 2, 2>(a, argv, G, nb, P, s);
    return launch_rs<64, 64, 2, 2>(a, argv, G, nb, P, s);
}

}  // namespace ens
