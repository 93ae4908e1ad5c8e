// The FC head of a bf16 member on the matrix cores: logits[n][co] = sum_k x[n][k] * W[k][co] + bias[co]
// with x the fp32 pooled features and W bf16.
//
// The pooled features stay fp32 (rounding them to bf16 would cost the logits three decimal digits):
// each value is split into two bf16 parts, hi = bf16(x) and lo = bf16(x - hi), and both parts go through
// the matrix cores against the same weight fragment.  Products of bf16 values are exact in fp32, so the
// result differs from the fp32 product sum by the 2^-17 of x that two bf16 parts do not hold.
//
// A workgroup owns 32 classes x 32 images; its four wavefronts split the K range and add their partial
// blocks up through LDS.  The weights come from a transposed copy in matrix-core operand order (1 KB in
// a row per wavefront and step), the features straight from memory, 32 bytes per lane and step.  A
// head of 2048 -> 1000 over 128 images is 128 workgroups that each read 0.4 MB: the kernel is a few
// microseconds of latency, where a kernel with one class per lane and eight images per workgroup spent
// 34 us streaming the weights sixteen times.
#include "conv_direct.h"

namespace ens {

__global__ __launch_bounds__(256) void fc_mfma_bf16(const FcArgs* __restrict__ argv, const int nb_, const long long first) {
    const FcArgs a = argv[blockIdx.z];
    __shared__ float red[3][16 * 64];
    const int t = threadIdx.x, lane = t & 63, lrow = lane & 31, lhalf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int c0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
    const int K = a.cin;
    const int NS = (K + 63) / 64 * 4;                // steps per block of 32 weight rows in the packed copy (columns padded to 64s)
    const int steps = (K + 15) / 16;                 // steps that hold features
    const int per = (steps + 3) / 4;
    const int s_begin = wave * per, s_end = min(steps, s_begin + per);

    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.wpk, 0, (int)((unsigned)((a.cout + 31) / 32) * (unsigned)NS * 1024u), 0x00020000);
    const unsigned wv = (unsigned)(blockIdx.x * NS * 1024 + lane * 16);
    const int n = n0 + lrow;
    const bool row_ok = n < nb_;
    // features through a buffer descriptor: rows past the batch and steps past K read zeros, so the loop has no branch
    // and the loads of several steps can be in flight together
    constexpr unsigned OOBV = 0x80000000u;
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc((void*)a.x, 0, (int)((unsigned)nb_ * (unsigned)K * 4u), 0x00020000);
    const unsigned xv = row_ok ? (unsigned)((n * K + 8 * lhalf) * 4) : OOBV;

    f32x16 acc;
    bn_zero(acc);
    auto step = [&](const bf16x8& wf, const f32x4& x0, const f32x4& x1) {
        const float xs[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int q = 0; q < 4; q++) {
            hi[q] = pack_bf16x2(xs[2 * q], xs[2 * q + 1]);
            const float r0 = xs[2 * q] - bf16_to_f32((uint16_t)(hi[q] & 0xFFFF));
            const float r1 = xs[2 * q + 1] - bf16_to_f32((uint16_t)(hi[q] >> 16));
            lo[q] = pack_bf16x2(r0, r1);
        }
        const bf16x8 xh = __builtin_bit_cast(bf16x8, u32x4{hi[0], hi[1], hi[2], hi[3]});
        const bf16x8 xl = __builtin_bit_cast(bf16x8, u32x4{lo[0], lo[1], lo[2], lo[3]});
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xh, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xl, acc, 0, 0, 0);
    };
    constexpr int U = 8;                             // steps whose loads are issued together
    for (int s0 = s_begin; s0 < s_end; s0 += U) {
        bf16x8 wf[U];
        f32x4 x0[U], x1[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int s = s0 + u;
            // a lane's 8 features of a step exist or do not (K is a multiple of 8); steps past this wave's share read nothing
            const bool live = s < s_end && 16 * s + 8 * lhalf + 8 <= K;
            wf[u] = bn_wload(wres, s < s_end ? wv : OOBV, s * 1024);
            x0[u] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(xres, live ? xv : OOBV, s * 64, 0));
            x1[u] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(xres, live ? xv : OOBV, s * 64 + 16, 0));
        }
#pragma unroll
        for (int u = 0; u < U; u++) step(wf[u], x0[u], x1[u]);
    }
    if (wave > 0) {
#pragma unroll
        for (int v = 0; v < 16; v++) red[wave - 1][v * 64 + lane] = acc[v];
    }
    __syncthreads();
    if (wave > 0 || !row_ok) return;
    // register v of a lane: class c0 + 16 (v / 8) + 8 (lane / 32) + v % 8 of image n0 + lane % 32
    float* __restrict__ y = a.y + (size_t)(first + n) * a.ldy;
#pragma unroll
    for (int v = 0; v < 16; v++) {
        const int co = c0 + 16 * (v / 8) + 8 * lhalf + (v % 8);
        if (co < a.cout) y[co] = acc[v] + red[0][v * 64 + lane] + red[1][v * 64 + lane] + red[2][v * 64 + lane] + a.bias[co];
    }
}

bool fc_mfma_applicable(const FcArgs& a) { return a.wpk != nullptr && a.cin % 8 == 0 && a.cin >= 64; }

hipError_t launch_fc_mfma(const FcArgs& a, const FcArgs* argv, int G, int nb, long long first, hipStream_t s) {
    if (!fc_mfma_applicable(a) || nb <= 0 || a.cout <= 0 || !a.bias || !a.y || !a.x || G <= 0 || !argv) return hipErrorInvalidValue;
    if ((long long)((a.cout + 31) / 32) * ((a.cin + 63) / 64 * 4) * 1024 >= 0x7FFFFF00LL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((a.cout + 31) / 32), (unsigned)((nb + 31) / 32), (unsigned)G);
    ENS_LAUNCH(fc_mfma_bf16, grid, dim3(256), 0, s, argv, nb, first);
    return hipGetLastError();
}

}  // namespace ens
