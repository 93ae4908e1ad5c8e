// Bandwidth-bound layers and the fp32 reference-precision convolution:
// input staging (convert / pad / bilinear resize), depthwise convolution, pooling, global
// average pool, squeeze-excite, the FC head and the fused softmax-and-mean combination.
// Activations are NHWC; the bf16 kernels move 8 channels (16 bytes) per lane so that a
// wavefront reads and writes whole 128-byte lines; all arithmetic is fp32.
#include "kernels.h"

namespace ens {

__device__ __forceinline__ float bf2f(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
// fp32 members: the exponential at full precision (the fast one is for results that are rounded to bf16)
__device__ __forceinline__ float act_f(float v, int act) {
    if (act == ACT_RELU) return fmaxf(v, 0.f);
    if (act == ACT_SILU) return v / (1.f + expf(-v));
    return v;
}
template <bool FAST>
__device__ __forceinline__ float exp_neg(float v) { return FAST ? __expf(-v) : expf(-v); }
// SiLU of a value that is rounded to bf16 afterwards: fast exponential, hardware reciprocal (an IEEE division is ten
// instructions, two of them at quarter rate, and the depthwise kernels are bound by the vector units)
__device__ __forceinline__ float silu_fast(float v) { return v * __builtin_amdgcn_rcpf(1.f + __expf(-v)); }
__device__ __forceinline__ void unpack8(const uint4 v, float* f) {
    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; e++) {
        f[2 * e] = bf2f((uint16_t)(u[e] & 0xFFFF));
        f[2 * e + 1] = bf2f((uint16_t)(u[e] >> 16));
    }
}
// f[e] = f[e] * scale[e] + bias[e] for 8 consecutive channels (16-byte aligned fp32 vectors)
__device__ __forceinline__ void scale_bias8(float* f, const float* scale, const float* bias) {
    const float4 s0 = *(const float4*)scale, s1 = *(const float4*)(scale + 4);
    const float4 b0 = *(const float4*)bias, b1 = *(const float4*)(bias + 4);
    f[0] = fmaf(f[0], s0.x, b0.x); f[1] = fmaf(f[1], s0.y, b0.y); f[2] = fmaf(f[2], s0.z, b0.z); f[3] = fmaf(f[3], s0.w, b0.w);
    f[4] = fmaf(f[4], s1.x, b1.x); f[5] = fmaf(f[5], s1.y, b1.y); f[6] = fmaf(f[6], s1.z, b1.z); f[7] = fmaf(f[7], s1.w, b1.w);
}

__device__ __forceinline__ uint4 pack8(const float* f) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    uint32_t u[4];
#pragma unroll
    for (int e = 0; e < 4; e++) {
        const f32x2_t v = {f[2 * e], f[2 * e + 1]};
        u[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));   // v_cvt_pk_bf16_f32, nearest even
    }
    return make_uint4(u[0], u[1], u[2], u[3]);
}

int& cu_budget() {
    static thread_local int units = 256;
    return units;
}

LaunchEvents& next_launch_events() {
    static thread_local LaunchEvents ev;
    return ev;
}

static inline int blocks_for(long long work, int threads) { return (int)((work + threads - 1) / threads); }

// ------------------------------------------------------------------ input staging
// Bilinear sample (half-pixel centres, edge clamp) of the three source channels at destination
// pixel (y, x) of a dh x dw image; a plain copy when the sizes agree.
__device__ __forceinline__ void stage_sample(const StageArgs& a, const float* __restrict__ src, int y, int x, float* v) {
    if (a.sh == a.dh && a.sw == a.dw) {
        const float* p = src + ((long long)y * a.sw + x) * 3;
        v[0] = p[0]; v[1] = p[1]; v[2] = p[2];
        return;
    }
    float fy = (y + 0.5f) * ((float)a.sh / (float)a.dh) - 0.5f;
    float fx = (x + 0.5f) * ((float)a.sw / (float)a.dw) - 0.5f;
    fy = fminf(fmaxf(fy, 0.f), (float)(a.sh - 1));
    fx = fminf(fmaxf(fx, 0.f), (float)(a.sw - 1));
    const int y0 = (int)floorf(fy), x0 = (int)floorf(fx);
    const int y1 = min(y0 + 1, a.sh - 1), x1 = min(x0 + 1, a.sw - 1);
    const float wy = fy - y0, wx = fx - x0;
#pragma unroll
    for (int c = 0; c < 3; c++) {
        const float p00 = src[((long long)y0 * a.sw + x0) * 3 + c], p01 = src[((long long)y0 * a.sw + x1) * 3 + c];
        const float p10 = src[((long long)y1 * a.sw + x0) * 3 + c], p11 = src[((long long)y1 * a.sw + x1) * 3 + c];
        const float top = p00 * (1.f - wx) + p01 * wx, bot = p10 * (1.f - wx) + p11 * wx;
        v[c] = top * (1.f - wy) + bot * wy;
    }
}

// One thread per destination pixel, written as dc channels (zero padded) in the member's dtype.
template <bool BF16>
__global__ void stage_kernel(const StageArgs* __restrict__ argv, const int nb_, const long long first) {
    StageArgs a = argv[blockIdx.z];
    a.nb = nb_;
    a.src += first * a.sh * a.sw * 3;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = (long long)a.nb * a.dh * a.dw;
    if (idx >= total) return;
    const int x = (int)(idx % a.dw);
    const int y = (int)((idx / a.dw) % a.dh);
    const long long n = idx / ((long long)a.dw * a.dh);
    const float* src = a.src + n * (long long)a.sh * a.sw * 3;
    float v[3];
    stage_sample(a, src, y, x, v);
    if (BF16) {
        uint16_t* d = (uint16_t*)a.dst + idx * a.dc;
        if (a.dc == 8) {
            const float f[8] = {v[0], v[1], v[2], 0.f, 0.f, 0.f, 0.f, 0.f};
            *(uint4*)d = pack8(f);
        } else {
            for (int c = 0; c < a.dc; c++) d[c] = c < 3 ? f2bf(v[c]) : (uint16_t)0;
        }
    } else {
        float* d = (float*)a.dst + idx * a.dc;
        for (int c = 0; c < a.dc; c++) d[c] = c < 3 ? v[c] : 0.f;
    }
}

// Space-to-depth staging (bf16): one thread per destination pixel (r, q) gathers the 2x2 image
// pixels (2r + by, 2q + bx) into channels (2*by + bx)*3 + c of a 16-channel pixel.
__global__ void stage_s2d_kernel(const StageArgs* __restrict__ argv, const int nb_, const long long first) {
    StageArgs a = argv[blockIdx.z];
    a.nb = nb_;
    a.src += first * a.sh * a.sw * 3;
    const int h2 = (a.dh + 1) / 2, w2 = (a.dw + 1) / 2;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = (long long)a.nb * h2 * w2;
    if (idx >= total) return;
    const int q = (int)(idx % w2);
    const int r = (int)((idx / w2) % h2);
    const long long n = idx / ((long long)w2 * h2);
    const float* src = a.src + n * (long long)a.sh * a.sw * 3;
    float f[16];
#pragma unroll
    for (int c = 0; c < 16; c++) f[c] = 0.f;
#pragma unroll
    for (int by = 0; by < 2; by++)
#pragma unroll
        for (int bx = 0; bx < 2; bx++) {
            const int y = 2 * r + by, x = 2 * q + bx;
            if (y < a.dh && x < a.dw) stage_sample(a, src, y, x, &f[(by * 2 + bx) * 3]);
        }
    uint4* d = (uint4*)((uint16_t*)a.dst + idx * 16);
    d[0] = pack8(f);
    d[1] = pack8(f + 8);
}

hipError_t launch_stage(const StageArgs& a, const StageArgs* argv, int G, int nb, long long first, bool bf16, hipStream_t s) {
    if (nb <= 0 || a.dc < 3 || G <= 0 || !argv) return hipErrorInvalidValue;
    if (a.s2d) {
        if (!bf16 || a.dc != 16) return hipErrorInvalidValue;
        const long long px = (long long)nb * ((a.dh + 1) / 2) * ((a.dw + 1) / 2);
        ENS_LAUNCH(stage_s2d_kernel, dim3(blocks_for(px, 256), 1, G), dim3(256), 0, s, argv, nb, first);
        return hipGetLastError();
    }
    const long long total = (long long)nb * a.dh * a.dw;
    const dim3 g(blocks_for(total, 256), 1, G);
    if (bf16) ENS_LAUNCH(stage_kernel<true>, g, dim3(256), 0, s, argv, nb, first);
    else ENS_LAUNCH(stage_kernel<false>, g, dim3(256), 0, s, argv, nb, first);
    return hipGetLastError();
}

// ------------------------------------------------------------------ fp32 convolution
// Reference-precision path (fp32 members): one thread per output element, taps and input
// channels accumulated in the order kh, kw, ci.  Weights [cout][kh][kw][cin] fp32.
__global__ void conv_f32_kernel(const ConvArgs* __restrict__ argv, const int nb_) {
    ConvArgs a = argv[blockIdx.z];
    a.nb = nb_;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = (long long)a.nb * a.Ho * a.Wo * a.cout;
    if (idx >= total) return;
    const int co = (int)(idx % a.cout);
    const long long p = idx / a.cout;
    const int wo = (int)(p % a.Wo), ho = (int)((p / a.Wo) % a.Ho);
    const long long n = p / ((long long)a.Wo * a.Ho);
    const float* x = (const float*)a.x.p + n * (long long)a.H * a.W * a.x.stride + a.x.c0;
    const float* w = (const float*)a.w + (long long)co * a.kh * a.kw * a.cin;
    float acc = 0.f;
    for (int kh = 0; kh < a.kh; kh++) {
        const int hi = ho * a.sh - a.pt + kh;
        if (hi < 0 || hi >= a.H) continue;
        for (int kw = 0; kw < a.kw; kw++) {
            const int wi = wo * a.sw - a.pl + kw;
            if (wi < 0 || wi >= a.W) continue;
            const float* px = x + ((long long)hi * a.W + wi) * a.x.stride;
            const float* wk = w + (kh * a.kw + kw) * a.cin;
            for (int ci = 0; ci < a.cin; ci++) {
                float v = px[ci];
                if (a.pre_scale) v = fmaxf(v * a.pre_scale[ci] + a.pre_shift[ci], 0.f);
                acc = fmaf(v, wk[ci], acc);
            }
        }
    }
    acc = fmaf(acc, a.scale[co], a.bias[co]);        // fp32 members: the scale is in the weights and this one is 1
    if (a.res.p) acc += ((const float*)a.res.p)[p * a.res.stride + a.res.c0 + co];
    ((float*)a.y.p)[p * a.y.stride + a.y.c0 + co] = act_f(acc, a.act);
}

hipError_t launch_conv_f32(const ConvArgs& a, const ConvArgs* argv, int G, int nb, hipStream_t s) {
    if (nb <= 0 || a.cin <= 0 || a.cout <= 0 || !a.bias || G <= 0 || !argv) return hipErrorInvalidValue;
    const long long total = (long long)nb * a.Ho * a.Wo * a.cout;
    if (total >= (1LL << 31) * 256) return hipErrorInvalidValue;
    ENS_LAUNCH(conv_f32_kernel, dim3(blocks_for(total, 256), 1, G), dim3(256), 0, s, argv, nb);
    return hipGetLastError();
}

// Windowed kernels (pooling, depthwise) read every input row for several output rows.  Consecutive
// workgroup ids go to different XCDs, each with its own L2; the ids are regrouped so that an XCD
// works on one contiguous run of the output and finds the shared input rows in its own L2.
__device__ __forceinline__ unsigned xcd_block() {
    const unsigned n = gridDim.x, b = blockIdx.x, per = n / 8;
    return b < per * 8 ? (b % 8) * per + b / 8 : b;
}

// ------------------------------------------------------------------ depthwise conv / pooling
// MODE 0: depthwise convolution (+bias, activation), 1: max pool, 2: average pool over the
// in-bounds part of the window.  bf16: one lane per (pixel, 8 channels); fp32: per element.
// The launcher admits fewer than 2^31 work items, so the index split runs in 32-bit arithmetic
// (64-bit division is a long instruction sequence); only the final element offsets are 64-bit.
template <int MODE, bool BF16>
__global__ void window_kernel(const PoolArgs* __restrict__ argv, const int nb_) {
    PoolArgs a = argv[blockIdx.z];
    a.nb = nb_;
    constexpr int V = BF16 ? 8 : 1;
    const unsigned cv = (unsigned)(a.c / V);
    const unsigned idx = xcd_block() * blockDim.x + threadIdx.x;
    const unsigned total = (unsigned)a.nb * (unsigned)(a.Ho * a.Wo) * cv;
    if (idx >= total) return;
    const unsigned pu = idx / cv;
    const int c = (int)(idx - pu * cv) * V;
    const unsigned row = pu / (unsigned)a.Wo;
    const int wo = (int)(pu - row * (unsigned)a.Wo);
    const unsigned nu = row / (unsigned)a.Ho;
    const int ho = (int)(row - nu * (unsigned)a.Ho);
    const long long p = pu, n = nu;
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; e++) acc[e] = MODE == 1 ? -3.0e38f : 0.f;
    int cnt = 0;
    for (int kh = 0; kh < a.kh; kh++) {
        const int hi = ho * a.sh - a.pt + kh;
        if (hi < 0 || hi >= a.H) continue;
        for (int kw = 0; kw < a.kw; kw++) {
            const int wi = wo * a.sw - a.pl + kw;
            if (wi < 0 || wi >= a.W) continue;
            const long long off = ((n * a.H + hi) * a.W + wi) * (long long)a.x.stride + a.x.c0 + c;
            float xv[V], wv[V];
            if (BF16) {
                unpack8(*(const uint4*)((const uint16_t*)a.x.p + off), xv);
                if (MODE == 0) unpack8(*(const uint4*)((const uint16_t*)a.w + (long long)(kh * a.kw + kw) * a.c + c), wv);
            } else {
                xv[0] = ((const float*)a.x.p)[off];
                if (MODE == 0) wv[0] = ((const float*)a.w)[(long long)(kh * a.kw + kw) * a.c + c];
            }
#pragma unroll
            for (int e = 0; e < V; e++) {
                if (MODE == 0) acc[e] = fmaf(xv[e], wv[e], acc[e]);
                else if (MODE == 1) acc[e] = fmaxf(acc[e], xv[e]);
                else acc[e] += xv[e];
            }
            cnt++;
        }
    }
    if (MODE == 0) {
        // one uniform branch for the launch's activation instead of a chain per value
#pragma unroll
        for (int e = 0; e < V; e++) acc[e] = fmaf(acc[e], a.scale[c + e], a.bias[c + e]);
        if (a.act == ACT_SILU) {
#pragma unroll
            for (int e = 0; e < V; e++) acc[e] = BF16 ? silu_fast(acc[e]) : acc[e] / (1.f + expf(-acc[e]));
        } else {
            const bool relu = a.act == ACT_RELU;
#pragma unroll
            for (int e = 0; e < V; e++) acc[e] = relu ? fmaxf(acc[e], 0.f) : acc[e];
        }
    } else {
#pragma unroll
        for (int e = 0; e < V; e++) {
            if (MODE == 2) acc[e] = cnt ? acc[e] / (float)cnt : 0.f;
            else if (cnt == 0) acc[e] = 0.f;
        }
    }
    const long long yoff = p * (long long)a.y.stride + a.y.c0 + c;
    if (BF16) *(uint4*)((uint16_t*)a.y.p + yoff) = pack8(acc);
    else ((float*)a.y.p)[yoff] = acc[0];
}

// Max pooling, bf16, one lane per (pixel, 8 channels).  Window positions outside the image are
// replaced by the nearest position inside it: that position belongs to the window too (a window
// the launcher admits overlaps the image), so the maximum is unchanged and all KH*KW loads are
// unconditional and in flight together.
template <int KH, int KW>
__global__ void maxpool_bf16_kernel(const PoolArgs* __restrict__ argv, const int nb_) {
    const PoolArgs a = argv[blockIdx.z];
    const unsigned cv = (unsigned)(a.c / 8);
    const unsigned idx = xcd_block() * blockDim.x + threadIdx.x;
    const unsigned total = (unsigned)nb_ * (unsigned)(a.Ho * a.Wo) * cv;
    if (idx >= total) return;
    const unsigned pu = idx / cv;
    const int c = (int)(idx - pu * cv) * 8;
    const unsigned row = pu / (unsigned)a.Wo;
    const int wo = (int)(pu - row * (unsigned)a.Wo);
    const unsigned nu = row / (unsigned)a.Ho;
    const int ho = (int)(row - nu * (unsigned)a.Ho);
    const uint16_t* __restrict__ x = (const uint16_t*)a.x.p + (long long)nu * a.H * a.W * a.x.stride + a.x.c0 + c;
    uint4 v[KH * KW];
#pragma unroll
    for (int kh = 0; kh < KH; kh++) {
        const int hi = min(max(ho * a.sh - a.pt + kh, 0), a.H - 1);
#pragma unroll
        for (int kw = 0; kw < KW; kw++) {
            const int wi = min(max(wo * a.sw - a.pl + kw, 0), a.W - 1);
            v[kh * KW + kw] = *(const uint4*)(x + (long long)(hi * a.W + wi) * a.x.stride);
        }
    }
    float acc[8], f[8];
    unpack8(v[0], acc);
#pragma unroll
    for (int k = 1; k < KH * KW; k++) {
        unpack8(v[k], f);
#pragma unroll
        for (int e = 0; e < 8; e++) acc[e] = fmaxf(acc[e], f[e]);
    }
    *(uint4*)((uint16_t*)a.y.p + (long long)pu * a.y.stride + a.y.c0 + c) = pack8(acc);
}

// Depthwise K x K convolution, bf16, one lane per (pixel, 8 channels).  Every tap is loaded from a
// position clamped into the image and zeroed by a select when the tap lies outside: the K
// activation loads and K weight loads of a filter row are unconditional and in flight together
// (the rows stay a loop: all K*K at once would spill registers).
template <int K>
__global__ void dwconv_bf16_kernel(const PoolArgs* __restrict__ argv, const int nb_) {
    const PoolArgs a = argv[blockIdx.z];
    const unsigned cv = (unsigned)(a.c / 8);
    const unsigned idx = xcd_block() * blockDim.x + threadIdx.x;
    const unsigned total = (unsigned)nb_ * (unsigned)(a.Ho * a.Wo) * cv;
    if (idx >= total) return;
    const unsigned pu = idx / cv;
    const int c = (int)(idx - pu * cv) * 8;
    const unsigned row = pu / (unsigned)a.Wo;
    const int wo = (int)(pu - row * (unsigned)a.Wo);
    const unsigned nu = row / (unsigned)a.Ho;
    const int ho = (int)(row - nu * (unsigned)a.Ho);
    const uint16_t* __restrict__ x = (const uint16_t*)a.x.p + (long long)nu * a.H * a.W * a.x.stride + a.x.c0 + c;
    const uint16_t* __restrict__ w = (const uint16_t*)a.w + c;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
    for (int kh = 0; kh < K; kh++) {
        const int hi = ho * a.sh - a.pt + kh;
        const bool hok = (unsigned)hi < (unsigned)a.H;
        const int hic = min(max(hi, 0), a.H - 1);
        uint4 xv[K], wv[K];
#pragma unroll
        for (int kw = 0; kw < K; kw++) {
            const int wic = min(max(wo * a.sw - a.pl + kw, 0), a.W - 1);
            xv[kw] = *(const uint4*)(x + (long long)(hic * a.W + wic) * a.x.stride);
            wv[kw] = *(const uint4*)(w + (kh * K + kw) * a.c);
        }
#pragma unroll
        for (int kw = 0; kw < K; kw++) {
            const bool ok = hok && (unsigned)(wo * a.sw - a.pl + kw) < (unsigned)a.W;
            if (!ok) xv[kw] = make_uint4(0u, 0u, 0u, 0u);
            float xf[8], wf[8];
            unpack8(xv[kw], xf);
            unpack8(wv[kw], wf);
#pragma unroll
            for (int e = 0; e < 8; e++) acc[e] = fmaf(xf[e], wf[e], acc[e]);
        }
    }
    scale_bias8(acc, a.scale + c, a.bias + c);
    if (a.act == ACT_SILU) {
#pragma unroll
        for (int e = 0; e < 8; e++) acc[e] = silu_fast(acc[e]);
    } else if (a.act == ACT_RELU) {
#pragma unroll
        for (int e = 0; e < 8; e++) acc[e] = fmaxf(acc[e], 0.f);
    }
    *(uint4*)((uint16_t*)a.y.p + (long long)pu * a.y.stride + a.y.c0 + c) = pack8(acc);
}

// Depthwise K x K convolution with stride S (the same both ways), bf16, one lane per (NW consecutive
// output columns, 8 channels).  With one output per lane every input value is fetched K x K times
// and the filter once per output, 2 K^2 loads of 16 bytes per 16 bytes stored, and the kernel is
// bound by the compute unit's 64 bytes per clock from L1, not by HBM.  Here a filter row costs
// (NW - 1) S + K input loads and K weight loads for NW outputs (K = 3, S = 1, NW = 4: 6.75 loads
// per output instead of 18).  Taps are loaded from positions clamped into the image and zeroed
// by a select when they lie outside; the filter rows stay a loop.
template <int K, int S, int NW>
__global__ __launch_bounds__(256) void dwconv_row_bf16_kernel(const PoolArgs* __restrict__ argv, const int nb_) {
    const PoolArgs a = argv[blockIdx.z];
    constexpr int NCOL = (NW - 1) * S + K;
    const unsigned cv = (unsigned)(a.c / 8);
    const unsigned wgroups = (unsigned)(a.Wo + NW - 1) / NW;     // lanes' runs of NW columns per output row
    const unsigned idx = xcd_block() * blockDim.x + threadIdx.x;
    const unsigned total = (unsigned)nb_ * (unsigned)a.Ho * wgroups * cv;
    if (idx >= total) return;
    const unsigned gu = idx / cv;
    const int c = (int)(idx - gu * cv) * 8;
    const unsigned row = gu / wgroups;                           // n * Ho + ho
    const int wo0 = (int)(gu - row * wgroups) * NW;
    const unsigned nu = row / (unsigned)a.Ho;
    const int ho = (int)(row - nu * (unsigned)a.Ho);
    const uint16_t* __restrict__ x = (const uint16_t*)a.x.p + (long long)nu * a.H * a.W * a.x.stride + a.x.c0 + c;
    const uint16_t* __restrict__ w = (const uint16_t*)a.w + c;
    float acc[NW][8];
#pragma unroll
    for (int o = 0; o < NW; o++)
#pragma unroll
        for (int e = 0; e < 8; e++) acc[o][e] = 0.f;
    const int wi0 = wo0 * S - a.pl;
#pragma unroll 1
    for (int kh = 0; kh < K; kh++) {
        const int hi = ho * S - a.pt + kh;
        const bool hok = (unsigned)hi < (unsigned)a.H;
        const int hic = min(max(hi, 0), a.H - 1);
        uint4 xv[NCOL], wv[K];
#pragma unroll
        for (int j = 0; j < NCOL; j++) {
            const int wic = min(max(wi0 + j, 0), a.W - 1);
            xv[j] = *(const uint4*)(x + (long long)(hic * a.W + wic) * a.x.stride);
        }
#pragma unroll
        for (int kw = 0; kw < K; kw++) wv[kw] = *(const uint4*)(w + (kh * K + kw) * a.c);
        float wf[K][8];
#pragma unroll
        for (int kw = 0; kw < K; kw++) unpack8(wv[kw], wf[kw]);
#pragma unroll
        for (int j = 0; j < NCOL; j++) {
            const bool ok = hok && (unsigned)(wi0 + j) < (unsigned)a.W;
            if (!ok) xv[j] = make_uint4(0u, 0u, 0u, 0u);
            float xf[8];
            unpack8(xv[j], xf);
            // input column j is tap kw = j - o S of output o
#pragma unroll
            for (int o = 0; o < NW; o++) {
                const int kw = j - o * S;
                if (kw >= 0 && kw < K) {
#pragma unroll
                    for (int e = 0; e < 8; e++) acc[o][e] = fmaf(xf[e], wf[kw][e], acc[o][e]);
                }
            }
        }
    }
    uint16_t* __restrict__ y = (uint16_t*)a.y.p + ((long long)row * a.Wo + wo0) * a.y.stride + a.y.c0 + c;
#pragma unroll
    for (int o = 0; o < NW; o++) {
        if (wo0 + o >= a.Wo) break;
        scale_bias8(acc[o], a.scale + c, a.bias + c);
        if (a.act == ACT_SILU) {
#pragma unroll
            for (int e = 0; e < 8; e++) acc[o][e] = silu_fast(acc[o][e]);
        } else if (a.act == ACT_RELU) {
#pragma unroll
            for (int e = 0; e < 8; e++) acc[o][e] = fmaxf(acc[o][e], 0.f);
        }
        *(uint4*)(y + (long long)o * a.y.stride) = pack8(acc[o]);
    }
}

// The depthwise convolution in front of a squeeze-excite block: dwconv_row_bf16_kernel, and each workgroup also
// leaves the channel sums of its outputs (of the rounded values, as the block's own summing kernel would read them)
// as one row of the block's scratch, so that the block does not read the tensor for them.  The workgroups of an
// image do not reach into the next one (`blocks` of them per image, the last one partly idle); a lane adds up
// its own outputs, the lanes of a workgroup that hold the same 8 channels are added through LDS in lane order,
// and every workgroup writes all c sums of its row (zeros for channels it holds no lane of): the order of every
// sum is fixed.
template <int K, int S, int NW>
__global__ __launch_bounds__(256) void dwconv_row_sum_bf16_kernel(const PoolArgs* __restrict__ argv, const int nb_, const int blocks) {
    const PoolArgs a = argv[blockIdx.z];
    constexpr int NCOL = (NW - 1) * S + K;
    __shared__ float red[256 * 8];
    const int t = threadIdx.x;
    const unsigned cv = (unsigned)(a.c / 8);
    const unsigned wgroups = (unsigned)(a.Wo + NW - 1) / NW;     // lanes' runs of NW columns per output row
    const unsigned wg = xcd_block();                             // workgroups regrouped per XCD, an image's side by side
    const unsigned nu = wg / (unsigned)blocks, blk = wg - nu * (unsigned)blocks;
    const unsigned items = (unsigned)a.Ho * wgroups * cv;        // (run of columns, 8 channels) pairs of one image
    const unsigned idx = blk * 256u + (unsigned)t;
    float sum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (idx < items) {
        const unsigned gu = idx / cv;
        const int c = (int)(idx - gu * cv) * 8;
        const int ho = (int)(gu / wgroups);
        const int wo0 = (int)(gu - (unsigned)ho * wgroups) * NW;
        const uint16_t* __restrict__ x = (const uint16_t*)a.x.p + (long long)nu * a.H * a.W * a.x.stride + a.x.c0 + c;
        const uint16_t* __restrict__ w = (const uint16_t*)a.w + c;
        float acc[NW][8];
#pragma unroll
        for (int o = 0; o < NW; o++)
#pragma unroll
            for (int e = 0; e < 8; e++) acc[o][e] = 0.f;
        const int wi0 = wo0 * S - a.pl;
#pragma unroll 1
        for (int kh = 0; kh < K; kh++) {
            const int hi = ho * S - a.pt + kh;
            const bool hok = (unsigned)hi < (unsigned)a.H;
            const int hic = min(max(hi, 0), a.H - 1);
            uint4 xv[NCOL], wv[K];
#pragma unroll
            for (int j = 0; j < NCOL; j++) {
                const int wic = min(max(wi0 + j, 0), a.W - 1);
                xv[j] = *(const uint4*)(x + (long long)(hic * a.W + wic) * a.x.stride);
            }
#pragma unroll
            for (int kw = 0; kw < K; kw++) wv[kw] = *(const uint4*)(w + (kh * K + kw) * a.c);
            float wf[K][8];
#pragma unroll
            for (int kw = 0; kw < K; kw++) unpack8(wv[kw], wf[kw]);
#pragma unroll
            for (int j = 0; j < NCOL; j++) {
                const bool ok = hok && (unsigned)(wi0 + j) < (unsigned)a.W;
                if (!ok) xv[j] = make_uint4(0u, 0u, 0u, 0u);
                float xf[8];
                unpack8(xv[j], xf);
#pragma unroll
                for (int o = 0; o < NW; o++) {
                    const int kw = j - o * S;                    // input column j is tap kw of output o
                    if (kw >= 0 && kw < K) {
#pragma unroll
                        for (int e = 0; e < 8; e++) acc[o][e] = fmaf(xf[e], wf[kw][e], acc[o][e]);
                    }
                }
            }
        }
        uint16_t* __restrict__ y = (uint16_t*)a.y.p + (((long long)nu * a.Ho + ho) * a.Wo + wo0) * a.y.stride + a.y.c0 + c;
#pragma unroll
        for (int o = 0; o < NW; o++) {
            if (wo0 + o >= a.Wo) break;
            scale_bias8(acc[o], a.scale + c, a.bias + c);
            if (a.act == ACT_SILU) {
#pragma unroll
                for (int e = 0; e < 8; e++) acc[o][e] = silu_fast(acc[o][e]);
            } else if (a.act == ACT_RELU) {
#pragma unroll
                for (int e = 0; e < 8; e++) acc[o][e] = fmaxf(acc[o][e], 0.f);
            }
            const uint4 packed = pack8(acc[o]);
            *(uint4*)(y + (long long)o * a.y.stride) = packed;
            float r[8];
            unpack8(packed, r);
#pragma unroll
            for (int e = 0; e < 8; e++) sum[e] += r[e];
        }
    }
#pragma unroll
    for (int e = 0; e < 8; e++) red[t * 8 + e] = sum[e];
    __syncthreads();
    float* out = a.sums + (long long)nu * a.sums_stride + (long long)blk * a.c;
    const unsigned shift = (blk * 256u) % cv;                    // lane t holds channel group (shift + t) mod cv
    for (unsigned g = (unsigned)t; g < cv; g += 256u) {
        float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (unsigned l = (g + cv - shift) % cv; l < 256u; l += cv)
#pragma unroll
            for (int e = 0; e < 8; e++) v[e] += red[l * 8 + e];
        *(float4*)(out + g * 8) = make_float4(v[0], v[1], v[2], v[3]);
        *(float4*)(out + g * 8 + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
}

// Average pooling over the in-bounds part of a K x K window, bf16, one lane per (pixel, 8
// channels): loads from clamped positions, taps outside the image zeroed by a select and left out
// of the divisor.
template <int K>
__global__ void avgpool_bf16_kernel(const PoolArgs* __restrict__ argv, const int nb_) {
    const PoolArgs a = argv[blockIdx.z];
    const unsigned cv = (unsigned)(a.c / 8);
    const unsigned idx = xcd_block() * blockDim.x + threadIdx.x;
    const unsigned total = (unsigned)nb_ * (unsigned)(a.Ho * a.Wo) * cv;
    if (idx >= total) return;
    const unsigned pu = idx / cv;
    const int c = (int)(idx - pu * cv) * 8;
    const unsigned row = pu / (unsigned)a.Wo;
    const int wo = (int)(pu - row * (unsigned)a.Wo);
    const unsigned nu = row / (unsigned)a.Ho;
    const int ho = (int)(row - nu * (unsigned)a.Ho);
    const uint16_t* __restrict__ x = (const uint16_t*)a.x.p + (long long)nu * a.H * a.W * a.x.stride + a.x.c0 + c;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; e++) acc[e] = 0.f;
    int cnt = 0;
    uint4 xv[K * K];
#pragma unroll
    for (int kh = 0; kh < K; kh++) {
        const int hic = min(max(ho * a.sh - a.pt + kh, 0), a.H - 1);
#pragma unroll
        for (int kw = 0; kw < K; kw++) {
            const int wic = min(max(wo * a.sw - a.pl + kw, 0), a.W - 1);
            xv[kh * K + kw] = *(const uint4*)(x + (long long)(hic * a.W + wic) * a.x.stride);
        }
    }
    // the pre-activation of a 1x1 convolution that lets this pool go first: relu(x * scale + shift) is averaged
    const bool pre = a.pre_scale != nullptr;
    float ps[8], pf[8];
    if (pre) {
        *(float4*)ps = *(const float4*)(a.pre_scale + c);
        *(float4*)(ps + 4) = *(const float4*)(a.pre_scale + c + 4);
        *(float4*)pf = *(const float4*)(a.pre_shift + c);
        *(float4*)(pf + 4) = *(const float4*)(a.pre_shift + c + 4);
    }
#pragma unroll
    for (int kh = 0; kh < K; kh++)
#pragma unroll
        for (int kw = 0; kw < K; kw++) {
            const bool ok = (unsigned)(ho * a.sh - a.pt + kh) < (unsigned)a.H && (unsigned)(wo * a.sw - a.pl + kw) < (unsigned)a.W;
            float f[8];
            unpack8(xv[kh * K + kw], f);
            if (pre) {
#pragma unroll
                for (int e = 0; e < 8; e++) f[e] = fmaxf(fmaf(f[e], ps[e], pf[e]), 0.f);
            }
            cnt += ok ? 1 : 0;
#pragma unroll
            for (int e = 0; e < 8; e++) acc[e] += ok ? f[e] : 0.f;
        }
    const float inv = cnt ? 1.f / (float)cnt : 0.f;
#pragma unroll
    for (int e = 0; e < 8; e++) acc[e] *= inv;
    // the activation of a 1x1 convolution that changed places with this pool
    if (a.act == ACT_RELU) {
#pragma unroll
        for (int e = 0; e < 8; e++) acc[e] = fmaxf(acc[e], 0.f);
    } else if (a.act == ACT_SILU) {
#pragma unroll
        for (int e = 0; e < 8; e++) acc[e] = silu_fast(acc[e]);
    }
    *(uint4*)((uint16_t*)a.y.p + (long long)pu * a.y.stride + a.y.c0 + c) = pack8(acc);
}

static hipError_t check_window(const PoolArgs& a, bool bf16) {
    if (a.c <= 0) return hipErrorInvalidValue;
    if (bf16 && (a.c % 8 || a.x.stride % 8 || a.x.c0 % 8 || a.y.stride % 8 || a.y.c0 % 8)) return hipErrorInvalidValue;
    return hipSuccess;
}

bool dwconv_sums_applicable(const PoolArgs& a, bool bf16) {
    const int st = a.sh == a.sw ? a.sh : 0;
    return bf16 && a.kh == a.kw && (a.kh == 3 || a.kh == 5) && (st == 1 || st == 2) && a.c % 8 == 0;
}

hipError_t launch_dwconv(const PoolArgs& a, const PoolArgs* argv, int G, int nb, bool bf16, hipStream_t s) {
    if (check_window(a, bf16) != hipSuccess || !a.w || !a.bias || !a.scale || nb <= 0 || G <= 0 || !argv) return hipErrorInvalidValue;
    const long long total = (long long)nb * a.Ho * a.Wo * (a.c / (bf16 ? 8 : 1));
    if (total >= (1LL << 31) - 256) return hipErrorInvalidValue;   // 32-bit work item index in the kernel
    const dim3 g(blocks_for(total, 256), 1, G);
    // 3x3 and 5x5 at strides 1 and 2: four output columns per lane (eight were measured too: no faster)
    const int st = a.sh == a.sw ? a.sh : 0;
    if (a.sums) {                                                // and a row of channel sums per workgroup
        if (!dwconv_sums_applicable(a, bf16) || a.sums_stride <= 0 || ((uintptr_t)a.sums & 15) || a.sums_stride % 4) return hipErrorInvalidValue;
        constexpr int NW = 4;
        const int blocks = dwconv_sums_blocks(a.Ho, a.Wo, a.c);
        if ((long long)blocks * nb >= (1LL << 31) / 256) return hipErrorInvalidValue;
        const dim3 gs((unsigned)(blocks * nb), 1, (unsigned)G);
        if (a.kh == 3 && st == 1) ENS_LAUNCH((dwconv_row_sum_bf16_kernel<3, 1, NW>), gs, dim3(256), 0, s, argv, nb, blocks);
        else if (a.kh == 3) ENS_LAUNCH((dwconv_row_sum_bf16_kernel<3, 2, NW>), gs, dim3(256), 0, s, argv, nb, blocks);
        else if (st == 1) ENS_LAUNCH((dwconv_row_sum_bf16_kernel<5, 1, NW>), gs, dim3(256), 0, s, argv, nb, blocks);
        else ENS_LAUNCH((dwconv_row_sum_bf16_kernel<5, 2, NW>), gs, dim3(256), 0, s, argv, nb, blocks);
        return hipGetLastError();
    }
    if (bf16 && a.kh == a.kw && (a.kh == 3 || a.kh == 5) && (st == 1 || st == 2)) {
        constexpr int NW = 4;
        const dim3 gw(blocks_for((long long)nb * a.Ho * ((a.Wo + NW - 1) / NW) * (a.c / 8), 256), 1, G);
        if (a.kh == 3 && st == 1) ENS_LAUNCH((dwconv_row_bf16_kernel<3, 1, NW>), gw, dim3(256), 0, s, argv, nb);
        else if (a.kh == 3) ENS_LAUNCH((dwconv_row_bf16_kernel<3, 2, NW>), gw, dim3(256), 0, s, argv, nb);
        else if (st == 1) ENS_LAUNCH((dwconv_row_bf16_kernel<5, 1, NW>), gw, dim3(256), 0, s, argv, nb);
        else ENS_LAUNCH((dwconv_row_bf16_kernel<5, 2, NW>), gw, dim3(256), 0, s, argv, nb);
        return hipGetLastError();
    }
    if (bf16 && a.kh == 3 && a.kw == 3) ENS_LAUNCH((dwconv_bf16_kernel<3>), g, dim3(256), 0, s, argv, nb);
    else if (bf16 && a.kh == 5 && a.kw == 5) ENS_LAUNCH((dwconv_bf16_kernel<5>), g, dim3(256), 0, s, argv, nb);
    else if (bf16) ENS_LAUNCH((window_kernel<0, true>), g, dim3(256), 0, s, argv, nb);
    else ENS_LAUNCH((window_kernel<0, false>), g, dim3(256), 0, s, argv, nb);
    return hipGetLastError();
}

hipError_t launch_pool(const PoolArgs& a, const PoolArgs* argv, int G, int nb, bool is_max, bool bf16, hipStream_t s) {
    if (check_window(a, bf16) != hipSuccess || nb <= 0 || G <= 0 || !argv) return hipErrorInvalidValue;
    const long long total = (long long)nb * a.Ho * a.Wo * (a.c / (bf16 ? 8 : 1));
    if (total >= (1LL << 31) - 256) return hipErrorInvalidValue;   // 32-bit work item index in the kernel
    const dim3 g(blocks_for(total, 256), 1, G), b(256);
    // only the two bf16 average-pool kernels apply an activation or a pre-activation
    if ((a.act != ACT_NONE || a.pre_scale) && (is_max || !bf16 || a.kh != a.kw || (a.kh != 3 && a.kh != 2))) return hipErrorInvalidValue;
    if ((a.pre_scale == nullptr) != (a.pre_shift == nullptr) || ((uintptr_t)a.pre_scale & 15) || ((uintptr_t)a.pre_shift & 15)) return hipErrorInvalidValue;
    if (is_max) {
        // every window must overlap the image for the clamped fast path (true for the padded layers of real networks)
        const bool overlap = a.pt < a.kh && a.pl < a.kw && (a.Ho - 1) * a.sh - a.pt < a.H && (a.Wo - 1) * a.sw - a.pl < a.W;
        if (bf16 && overlap && a.kh == 3 && a.kw == 3) ENS_LAUNCH((maxpool_bf16_kernel<3, 3>), g, b, 0, s, argv, nb);
        else if (bf16 && overlap && a.kh == 2 && a.kw == 2) ENS_LAUNCH((maxpool_bf16_kernel<2, 2>), g, b, 0, s, argv, nb);
        else if (bf16) ENS_LAUNCH((window_kernel<1, true>), g, b, 0, s, argv, nb);
        else ENS_LAUNCH((window_kernel<1, false>), g, b, 0, s, argv, nb);
    } else {
        if (bf16 && a.kh == 3 && a.kw == 3) ENS_LAUNCH((avgpool_bf16_kernel<3>), g, b, 0, s, argv, nb);
        else if (bf16 && a.kh == 2 && a.kw == 2) ENS_LAUNCH((avgpool_bf16_kernel<2>), g, b, 0, s, argv, nb);
        else if (bf16) ENS_LAUNCH((window_kernel<2, true>), g, b, 0, s, argv, nb);
        else ENS_LAUNCH((window_kernel<2, false>), g, b, 0, s, argv, nb);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ global average pool
// A workgroup owns one image and 32 channel groups (16-byte groups of 8 channels for bf16): lanes
// run along the channels so that every pixel row is read in whole lines, the pixels are dealt
// round-robin to 8 thread rows (a 7x7 map: six or seven independent loads per thread, where one
// workgroup per image walked 49 pixels one after the other) and the partial sums are added
// through LDS in a fixed order.
constexpr int GAP_COLS = 32, GAP_ROWS = 8;
template <bool BF16>
__global__ __launch_bounds__(256) void gap_kernel(const GapArgs* __restrict__ argv, const int nb_) {
    GapArgs a = argv[blockIdx.z];
    a.nb = nb_;
    constexpr int V = BF16 ? 8 : 1;
    __shared__ float part[256 * V];
    const int n = blockIdx.x;
    const int cv = (a.c + V - 1) / V;                 // channel groups
    // 32 channel groups side by side, 8 pixel phases: a thread's loads are few and independent
    const int col = threadIdx.x % GAP_COLS, row = threadIdx.x / GAP_COLS;
    const int g = blockIdx.y * GAP_COLS + col;
    const bool pre = a.pre_scale != nullptr;
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; e++) acc[e] = 0.f;
    if (g < cv) {
        const int c = g * V;
        float sc[V], sf[V];
#pragma unroll
        for (int e = 0; e < V; e++) {
            sc[e] = pre && c + e < a.c ? a.pre_scale[c + e] : 1.f;
            sf[e] = pre && c + e < a.c ? a.pre_shift[c + e] : 0.f;
        }
#pragma unroll 4
        for (int p = row; p < a.HW; p += GAP_ROWS) {
            const long long off = ((long long)n * a.HW + p) * a.x.stride + a.x.c0 + c;
            float v[V];
            if (BF16) unpack8(*(const uint4*)((const uint16_t*)a.x.p + off), v);
            else v[0] = ((const float*)a.x.p)[off];
#pragma unroll
            for (int e = 0; e < V; e++) acc[e] += pre ? fmaxf(v[e] * sc[e] + sf[e], 0.f) : v[e];
        }
    }
#pragma unroll
    for (int e = 0; e < V; e++) part[threadIdx.x * V + e] = acc[e];
    __syncthreads();
    if (row == 0 && g < cv) {
#pragma unroll
        for (int e = 0; e < V; e++) {
            float s = 0.f;
#pragma unroll
            for (int r = 0; r < GAP_ROWS; r++) s += part[(r * GAP_COLS + col) * V + e];
            if (g * V + e < a.c) a.y[(long long)n * a.c + g * V + e] = s / (float)a.HW;
        }
    }
}

hipError_t launch_gap(const GapArgs& a, const GapArgs* argv, int G, int nb, bool bf16, hipStream_t s) {
    if (nb <= 0 || a.c <= 0 || a.HW <= 0 || G <= 0 || !argv) return hipErrorInvalidValue;
    if (bf16 && (a.c % 8 || a.x.stride % 8 || a.x.c0 % 8)) return hipErrorInvalidValue;
    const int cv = bf16 ? (a.c + 7) / 8 : a.c;
    const dim3 grid(nb, (cv + GAP_COLS - 1) / GAP_COLS, G);
    if (bf16) ENS_LAUNCH(gap_kernel<true>, grid, dim3(256), 0, s, argv, nb);
    else ENS_LAUNCH(gap_kernel<false>, grid, dim3(256), 0, s, argv, nb);
    return hipGetLastError();
}

// ------------------------------------------------------------------ FC head
// A workgroup owns 64 classes and up to 8 images.  The pooled features of those images sit in
// LDS; each of the four wavefronts walks a quarter of the input features with its lanes along
// the classes (coalesced weight rows, every weight used for all 8 images), and the four partial
// sums meet in LDS.
constexpr int FC_IMGS = 8;
constexpr int FC_KCH = 1024;       // input features staged in LDS at a time

constexpr int FC_WAVES = 16;       // waves per workgroup: each takes 1/16 of the K range of a chunk
template <bool BF16>
__global__ __launch_bounds__(FC_WAVES * 64) void fc_kernel(const FcArgs* __restrict__ argv, const int nb_, const long long first) {
    FcArgs a = argv[blockIdx.z];
    a.nb = nb_;
    a.y += first * a.ldy;
    __shared__ float xs[FC_IMGS * FC_KCH];
    __shared__ float part[FC_WAVES * FC_IMGS * 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int co = blockIdx.x * 64 + lane;
    const int n0 = blockIdx.y * FC_IMGS;
    const int ni = min(FC_IMGS, a.nb - n0);
    float acc[FC_IMGS];
#pragma unroll
    for (int e = 0; e < FC_IMGS; e++) acc[e] = 0.f;
    for (int kc = 0; kc < a.cin; kc += FC_KCH) {
        const int kn = min(FC_KCH, a.cin - kc);
        for (int i = threadIdx.x; i < FC_IMGS * kn; i += FC_WAVES * 64) {
            const int img = i / kn, k = i - img * kn;
            xs[img * FC_KCH + k] = img < ni ? a.x[(long long)(n0 + img) * a.cin + kc + k] : 0.f;
        }
        __syncthreads();
        const int per = (kn + FC_WAVES - 1) / FC_WAVES;
        const int k0 = wave * per, k1 = min(kn, k0 + per);
        if (co < a.cout) {
            // the weight loads of a wave are independent: many in flight hide the memory latency
#pragma unroll 16
            for (int k = k0; k < k1; k++) {
                const long long off = (long long)(kc + k) * a.cout + co;
                const float w = BF16 ? bf2f(((const uint16_t*)a.w)[off]) : ((const float*)a.w)[off];
#pragma unroll
                for (int e = 0; e < FC_IMGS; e++) acc[e] = fmaf(xs[e * FC_KCH + k], w, acc[e]);
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int e = 0; e < FC_IMGS; e++) part[(wave * FC_IMGS + e) * 64 + lane] = acc[e];
    __syncthreads();
    for (int i = threadIdx.x; i < FC_IMGS * 64; i += FC_WAVES * 64) {
        const int e = i >> 6, l = i & 63;
        const int c = blockIdx.x * 64 + l;
        if (e < ni && c < a.cout) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < FC_WAVES; w++) s += part[(w * FC_IMGS + e) * 64 + l];
            a.y[(long long)(n0 + e) * a.ldy + c] = s + a.bias[c];
        }
    }
}

hipError_t launch_fc(const FcArgs& a, const FcArgs* argv, int G, int nb, long long first, bool bf16, hipStream_t s) {
    if (nb <= 0 || a.cin <= 0 || a.cout <= 0 || !a.bias || !a.y || G <= 0 || !argv) return hipErrorInvalidValue;
    if (bf16 && fc_mfma_applicable(a)) return launch_fc_mfma(a, argv, G, nb, first, s);
    const dim3 g((a.cout + 63) / 64, (nb + FC_IMGS - 1) / FC_IMGS, G), b(FC_WAVES * 64);
    if (bf16) ENS_LAUNCH(fc_kernel<true>, g, b, 0, s, argv, nb, first);
    else ENS_LAUNCH(fc_kernel<false>, g, b, 0, s, argv, nb, first);
    return hipGetLastError();
}

// ------------------------------------------------------------------ squeeze-excite
// Two kernels on the worker's stream.  (1) Channel sums: workgroup (split, image) adds its share
// of the image's pixels; lanes run along the channels (16-byte groups of 8 for bf16) so that every
// pixel is read in whole lines, the pixels of the share are dealt round-robin to the thread rows
// and the rows are added through LDS.  (2) Gate and rescale: a workgroup adds the partial sums of
// its image, runs the two small FC layers (SiLU, sigmoid) and rescales its share of the image.
// Workgroups that share an image's pixels in the channel sums: one per 512 pixels, more when the
// launch would otherwise have fewer than about 2048 workgroups (small maps, small batches), never
// fewer than 8 pixels each.
static inline int se_splits(int HW, int images) {
    int s = (HW + 511) / 512;
    const int fill = (2048 + images - 1) / (images > 0 ? images : 1);
    if (s < fill) s = fill;
    if (s > HW / 8) s = HW / 8;
    return s < 1 ? 1 : (s > SE_MAX_SPLITS ? SE_MAX_SPLITS : s);
}

template <bool BF16>
__global__ __launch_bounds__(256) void se_sum_kernel(const SeArgs* __restrict__ argv, const int nb_) {
    const SeArgs a = argv[blockIdx.z];
    constexpr int V = BF16 ? 8 : 1;
    __shared__ float part[256 * V];
    const int split = blockIdx.x, n = blockIdx.y, splits = gridDim.x;
    const int chunk = (a.HW + splits - 1) / splits;
    const int p0 = split * chunk, p1 = min(a.HW, p0 + chunk);
    const int cv = (a.c + V - 1) / V;                 // channel groups
    const int cols = min(cv, 256);                    // groups handled side by side
    const int rows = 256 / cols;                      // pixel phases
    const int col = threadIdx.x % cols, row = threadIdx.x / cols;
    float* out = a.scratch + (long long)n * se_scratch_floats(a.c, a.r, a.cap) + (long long)split * a.c;
    for (int g0 = 0; g0 < cv; g0 += cols) {
        const int g = g0 + col;
        float acc[V];
#pragma unroll
        for (int e = 0; e < V; e++) acc[e] = 0.f;
        if (g < cv && row < rows) {
            const long long base = (long long)n * a.HW * a.x.stride + a.x.c0 + g * V;
            // four loads in flight per lane; the sums keep the order of the pixels
            for (int p = p0 + row; p < p1; p += 4 * rows) {
                float v[4][V];
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    const int pu = min(p + u * rows, p1 - 1);
                    const long long off = base + (long long)pu * a.x.stride;
                    if (BF16) unpack8(*(const uint4*)((const uint16_t*)a.x.p + off), v[u]);
                    else v[u][0] = ((const float*)a.x.p)[off];
                }
#pragma unroll
                for (int u = 0; u < 4; u++)
                    if (p + u * rows < p1) {
#pragma unroll
                        for (int e = 0; e < V; e++) acc[e] += v[u][e];
                    }
            }
        }
#pragma unroll
        for (int e = 0; e < V; e++) part[threadIdx.x * V + e] = acc[e];
        __syncthreads();
        if (row == 0 && g < cv) {
#pragma unroll
            for (int e = 0; e < V; e++) {
                float s = 0.f;
                for (int r = 0; r < rows; r++) s += part[(r * cols + col) * V + e];
                if (g * V + e < a.c) out[g * V + e] = s;
            }
        }
        __syncthreads();
    }
}

constexpr int SE_GATE_THREADS = 1024;   // the gate is a chain of dependent memory latencies: many threads, few steps each
constexpr int SE_GATE_MAXC = 4096;      // channels the gate holds in LDS
constexpr int SE_SCALE_BYTES = 32768;   // about what a workgroup of the last kernel rescales

// The gate of image n into LDS (`gate`): the partial sums added in a fixed order, then the two
// small FC layers (SiLU, sigmoid) with all threads on the first one.
template <bool FAST>
__device__ __forceinline__ void se_gate(const SeArgs& a, const int n, const int splits, float* mean, float* red, float* z, float* gate) {
    const int t = threadIdx.x;
    // Every loop below asks for a batch of values before it uses the first: a round trip to memory is about
    // 2000 clocks, and taken one load at a time the sums, the two weight matrices and the biases were some
    // thirty of them in a row (18 us per launch for a few ten thousand multiply-adds).
    const float* part = a.scratch + (long long)n * se_scratch_floats(a.c, a.r, a.cap);   // partial sums of the image
    const float inv = 1.f / (float)a.HW;
    for (int c = t; c < a.c; c += SE_GATE_THREADS) {
        float m = 0.f;
        for (int k0 = 0; k0 < splits; k0 += SE_MAX_SPLITS) {     // sixteen rows at a time; the summing depthwise kernel leaves more than that
            float v[SE_MAX_SPLITS];
#pragma unroll
            for (int k = 0; k < SE_MAX_SPLITS; k++) v[k] = k0 + k < splits ? part[(long long)(k0 + k) * a.c + c] : 0.f;
#pragma unroll
            for (int k = 0; k < SE_MAX_SPLITS; k++) m += v[k];   // fixed order; the terms past the last row are zeros
        }
        mean[c] = m * inv;
    }
    __syncthreads();
    // hidden layer: thread (slice, r) adds its slice of the channels; adjacent threads read adjacent weights
    int rp = 1;
    while (rp < a.r && rp < 256) rp <<= 1;
    const int slices = SE_GATE_THREADS / rp;
    for (int r0 = 0; r0 < a.r; r0 += rp) {
        const int r = r0 + t % rp, slice = t / rp;
        float acc = 0.f;
        if (r < a.r) {
            constexpr int U = 16;
            for (int c0 = slice; c0 < a.c; c0 += slices * U) {
                float w[U];
#pragma unroll
                for (int u = 0; u < U; u++) {
                    const int c = c0 + u * slices;
                    w[u] = c < a.c ? a.w1[(long long)c * a.r + r] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < U; u++) {
                    const int c = c0 + u * slices;
                    acc = fmaf(c < a.c ? mean[c] : 0.f, w[u], acc);
                }
            }
        }
        red[t] = acc;
        __syncthreads();
        if (t < rp && r < a.r) {
            float sum = a.b1[r];
            for (int k = 0; k < slices; k++) sum += red[k * rp + t];
            z[r] = sum / (1.f + exp_neg<FAST>(sum));
        }
        __syncthreads();
    }
    for (int c = t; c < a.c; c += SE_GATE_THREADS) {
        float acc = a.b2[c];
        constexpr int U = 16;
        for (int r0 = 0; r0 < a.r; r0 += U) {
            float w[U];
#pragma unroll
            for (int u = 0; u < U; u++) w[u] = r0 + u < a.r ? a.w2[(long long)(r0 + u) * a.c + c] : 0.f;
#pragma unroll
            for (int u = 0; u < U; u++) acc = fmaf(r0 + u < a.r ? z[r0 + u] : 0.f, w[u], acc);
        }
        gate[c] = 1.f / (1.f + exp_neg<FAST>(acc));
    }
    __syncthreads();
}

// Gate and rescale in one kernel: workgroup (share, image) works out the image's gate (every share of
// an image does, from the same sums in the same order: the two FC layers are a few ten thousand
// multiply-adds, a launch of their own cost 13 us) and rescales its share of the image's pixels.
template <bool BF16>
__global__ __launch_bounds__(SE_GATE_THREADS) void se_gate_scale_kernel(const SeArgs* __restrict__ argv, const int nb_, const int splits) {
    const SeArgs a = argv[blockIdx.z];
    __shared__ float mean[SE_GATE_MAXC];
    __shared__ __attribute__((aligned(16))) float gate[SE_GATE_MAXC];
    __shared__ float red[SE_GATE_THREADS];
    __shared__ float z[256];
    const int n = blockIdx.y;
    se_gate<BF16>(a, n, splits, mean, red, z, gate);
    constexpr int V = BF16 ? 8 : 1;
    const int cv = a.c / V;
    const int per = (a.HW + (int)gridDim.x - 1) / (int)gridDim.x;
    const int p0 = blockIdx.x * per, p1 = min(a.HW, p0 + per);
    const int items = p1 > p0 ? (p1 - p0) * cv : 0;
    for (int i = threadIdx.x; i < items; i += SE_GATE_THREADS) {
        const int q = i / cv, c = (i - q * cv) * V;
        const long long pix = (long long)n * a.HW + p0 + q;
        const long long xo = pix * a.x.stride + a.x.c0 + c, yo = pix * a.y.stride + a.y.c0 + c;
        if (BF16) {
            float f[8];
            unpack8(*(const uint4*)((const uint16_t*)a.x.p + xo), f);
            const float4 g0 = *(const float4*)&gate[c], g1 = *(const float4*)&gate[c + 4];
            f[0] *= g0.x; f[1] *= g0.y; f[2] *= g0.z; f[3] *= g0.w;
            f[4] *= g1.x; f[5] *= g1.y; f[6] *= g1.z; f[7] *= g1.w;
            *(uint4*)((uint16_t*)a.y.p + yo) = pack8(f);
        } else {
            ((float*)a.y.p)[yo] = ((const float*)a.x.p)[xo] * gate[c];
        }
    }
}

// The gates alone, one workgroup per image, into the image's scratch: for a squeeze-excite whose consumer
// (a 1x1 convolution) multiplies its input by them, so that the rescaled tensor is never written.
__global__ __launch_bounds__(SE_GATE_THREADS) void se_gate_only_kernel(const SeArgs* __restrict__ argv, const int nb_, const int splits) {
    const SeArgs a = argv[blockIdx.z];
    __shared__ float mean[SE_GATE_MAXC];
    __shared__ __attribute__((aligned(16))) float gate[SE_GATE_MAXC];
    __shared__ float red[SE_GATE_THREADS];
    __shared__ float z[256];
    const int n = blockIdx.y;
    se_gate<true>(a, n, splits, mean, red, z, gate);        // bf16 members only
    float* out = a.scratch + (long long)n * se_scratch_floats(a.c, a.r, a.cap) + se_gate_offset(a.c, a.r, a.cap);
    for (int c = threadIdx.x; c < a.c; c += SE_GATE_THREADS) out[c] = gate[c];
}

hipError_t launch_se(const SeArgs& a, const SeArgs* argv, int G, int nb, bool bf16, hipStream_t s) {
    if (nb <= 0 || a.c <= 0 || a.r <= 0 || a.HW <= 0 || !a.scratch || G <= 0 || !argv) return hipErrorInvalidValue;
    if (a.c > SE_GATE_MAXC || a.r > 256) return hipErrorInvalidValue;   // what the gate kernel holds in LDS
    if (bf16 && (a.c % 8 || a.x.stride % 8 || a.x.c0 % 8 || a.y.stride % 8 || a.y.c0 % 8)) return hipErrorInvalidValue;
    if ((long long)nb * a.HW >= (1LL << 31) / 8) return hipErrorInvalidValue;
    if (a.cap < SE_MAX_SPLITS || a.have_sums > a.cap || (a.have_sums && !bf16)) return hipErrorInvalidValue;
    const int splits = a.have_sums > 0 ? a.have_sums : se_splits(a.HW, nb * G);
    if (a.have_sums > 0) {}                                      // the kernel that wrote x has left the rows of partial sums
    else if (bf16) ENS_LAUNCH_FIRST(se_sum_kernel<true>, dim3(splits, nb, G), dim3(256), 0, s, argv, nb);
    else ENS_LAUNCH_FIRST(se_sum_kernel<false>, dim3(splits, nb, G), dim3(256), 0, s, argv, nb);
    if (a.gate_only) {
        if (a.have_sums > 0) ENS_LAUNCH(se_gate_only_kernel, dim3(1, nb, G), dim3(SE_GATE_THREADS), 0, s, argv, nb, splits);
        else ENS_LAUNCH_LAST(se_gate_only_kernel, dim3(1, nb, G), dim3(SE_GATE_THREADS), 0, s, argv, nb, splits);
        return hipGetLastError();
    }
    // shares of an image in the second kernel: about SE_SCALE_BYTES of the tensor each
    long long shares = ((long long)a.HW * a.c * (bf16 ? 2 : 4) + SE_SCALE_BYTES - 1) / SE_SCALE_BYTES;
    // and no more workgroups than the chip holds at once (two of 1024 threads per compute unit): every
    // workgroup starts with the gate's chain of memory latencies, which a second round would pay again
    const long long room = 512 / ((long long)nb * G);
    if (shares > room) shares = room;
    if (shares > a.HW) shares = a.HW;
    if (shares < 1) shares = 1;
    if (a.have_sums > 0) ENS_LAUNCH(se_gate_scale_kernel<true>, dim3((unsigned)shares, nb, G), dim3(SE_GATE_THREADS), 0, s, argv, nb, splits);
    else if (bf16) ENS_LAUNCH_LAST(se_gate_scale_kernel<true>, dim3((unsigned)shares, nb, G), dim3(SE_GATE_THREADS), 0, s, argv, nb, splits);
    else ENS_LAUNCH_LAST(se_gate_scale_kernel<false>, dim3((unsigned)shares, nb, G), dim3(SE_GATE_THREADS), 0, s, argv, nb, splits);
    return hipGetLastError();
}

// ------------------------------------------------------------------ combination rule
// One wavefront per sample: for each member a max-subtracted softmax of its logits row
// (wavefront shuffles for the maximum and the sum), each term divided by M and added in
// member order, one write of the combined row.
constexpr int COMBINE_MAX_PER_LANE = 32;    // classes <= 64 * 32

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

template <int PER, int RULE>
__global__ __launch_bounds__(256) void combine_kernel(const float* const* logits, const float* __restrict__ weights,
                                                      int n_members, long long n, int classes, float* y) {
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= n) return;
    float acc[PER];
#pragma unroll
    for (int e = 0; e < PER; e++) acc[e] = 0.f;
    const float inv_m = 1.f / (float)n_members;
    for (int m = 0; m < n_members; m++) {
        const float* z = logits[m] + row * classes;
        float v[PER];
        float mx = -3.0e38f;
        int arg = 0x7FFFFFFF;                        // class of this lane's maximum, lowest index first
#pragma unroll
        for (int e = 0; e < PER; e++) {
            const int c = lane + 64 * e;
            v[e] = c < classes ? z[c] : -3.0e38f;
            if (RULE == COMBINE_VOTE && c < classes && (v[e] > mx || arg == 0x7FFFFFFF)) arg = c;
            mx = fmaxf(mx, v[e]);
        }
        if (RULE == COMBINE_VOTE) {
            // arg-max over the wave: the larger value wins, the lower class on equal values
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                const float om = __shfl_xor(mx, off, 64);
                const int oa = __shfl_xor(arg, off, 64);
                if (om > mx || (om == mx && oa < arg)) { mx = om; arg = oa; }
            }
#pragma unroll
            for (int e = 0; e < PER; e++) acc[e] += lane + 64 * e == arg ? inv_m : 0.f;
            continue;
        }
        mx = wave_max(mx);
        float sum = 0.f;
#pragma unroll
        for (int e = 0; e < PER; e++) {
            const int c = lane + 64 * e;
            v[e] = c < classes ? expf(v[e] - mx) : 0.f;
            sum += v[e];
        }
        sum = wave_sum(sum);
        const float wm = RULE == COMBINE_WEIGHTED ? weights[m] : inv_m;
#pragma unroll
        for (int e = 0; e < PER; e++) acc[e] += (v[e] / sum) * wm;
    }
#pragma unroll
    for (int e = 0; e < PER; e++) {
        const int c = lane + 64 * e;
        if (c < classes) y[row * classes + c] = acc[e];
    }
}

template <int RULE>
static void launch_combine_rule(const float* const* logits, const float* weights, int n_members, int64_t n, int classes,
                                float* y, hipStream_t s) {
    const dim3 g((unsigned)((n + 3) / 4)), b(256);
    const int per = (classes + 63) / 64;
    if (per <= 1) ENS_LAUNCH((combine_kernel<1, RULE>), g, b, 0, s, logits, weights, n_members, (long long)n, classes, y);
    else if (per <= 4) ENS_LAUNCH((combine_kernel<4, RULE>), g, b, 0, s, logits, weights, n_members, (long long)n, classes, y);
    else if (per <= 16) ENS_LAUNCH((combine_kernel<16, RULE>), g, b, 0, s, logits, weights, n_members, (long long)n, classes, y);
    else ENS_LAUNCH((combine_kernel<32, RULE>), g, b, 0, s, logits, weights, n_members, (long long)n, classes, y);
}

hipError_t launch_combine(const float* const* logits, const float* weights, int rule, int n_members, int64_t n,
                          int classes, float* y, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    if (n_members <= 0 || classes <= 0 || classes > 64 * COMBINE_MAX_PER_LANE) return hipErrorInvalidValue;
    if (rule == COMBINE_MEAN) launch_combine_rule<COMBINE_MEAN>(logits, weights, n_members, n, classes, y, s);
    else if (rule == COMBINE_WEIGHTED && weights) launch_combine_rule<COMBINE_WEIGHTED>(logits, weights, n_members, n, classes, y, s);
    else if (rule == COMBINE_VOTE) launch_combine_rule<COMBINE_VOTE>(logits, weights, n_members, n, classes, y, s);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------ calibration images
// Content does not matter for classification throughput (section "Offline benchmark settings",
// "Calibration data samples"): hashed values uniform in [-1.73, 1.73) (unit variance).
__global__ void fill_noise_kernel(float* p, long long count, unsigned long long seed) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    unsigned long long z = seed + (unsigned long long)(i + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    p[i] = ((float)(z >> 40) * (1.0f / 16777216.0f) - 0.5f) * 3.4641016f;
}

__global__ void fill_zero_kernel(float* __restrict__ p, long long count) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0.f;
}

hipError_t launch_fill_zero(float* p, int64_t count, hipStream_t s) {
    if (count <= 0) return hipSuccess;
    ENS_LAUNCH(fill_zero_kernel, dim3(blocks_for(count, 256)), dim3(256), 0, s, p, (long long)count);
    return hipGetLastError();
}

hipError_t launch_fill_noise(float* p, int64_t count, uint64_t seed, hipStream_t s) {
    if (count <= 0) return hipSuccess;
    ENS_LAUNCH(fill_noise_kernel, dim3(blocks_for(count, 256)), dim3(256), 0, s, p, (long long)count,
                       (unsigned long long)seed);
    return hipGetLastError();
}

}  // namespace ens
