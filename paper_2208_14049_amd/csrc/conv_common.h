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
// SiLU of a value that is rounded to bf16 afterwards: the fast exponential and the hardware reciprocal (1 ulp each in
// fp32, against a rounding step of 2^-9).  An IEEE division is a sequence of ten instructions, two of them at quarter
// rate: with it the epilogues of layers that write several times what they read were bound by the vector units.
__device__ __forceinline__ float silu_bf16(float v) { return v * __builtin_amdgcn_rcpf(1.f + __expf(-v)); }

// Activation of N values at once.  `act` is the same for the whole launch: one uniform three-way
// branch per call instead of a chain of branches (or a select) per value.
template <int N>
__device__ __forceinline__ void apply_act_n(float* v, int act) {
    if (act == ACT_RELU) {
#pragma unroll
        for (int i = 0; i < N; i++) v[i] = fmaxf(v[i], 0.f);
    } else if (act == ACT_SILU) {
#pragma unroll
        for (int i = 0; i < N; i++) v[i] = silu_bf16(v[i]);
    }
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

// Share of the n_tiles position tiles that a persistent workgroup walks: tiles first, first + step, ...
// below end.  Consecutive workgroup ids go to different XCDs; the tiles are cut into 8 runs, one per
// XCD, and the workgroups of an XCD stride through its run, so that neighbouring tiles, whose input
// windows overlap, are fetched into one L2.  lin0: linear id of the workgroup with blockIdx.x == 0
// in this (y, z) plane of the grid.
struct TileWalk { int first, step, end; };
__device__ __forceinline__ TileWalk tile_walk(int n_tiles, int lin0) {
    TileWalk w;
    const int nx = gridDim.x, x = blockIdx.x;
    if (nx < 8) {
        w.first = x; w.step = nx; w.end = n_tiles;
        return w;
    }
    const int xcd = (lin0 + x) & 7;
    const int xfirst = (xcd - lin0) & 7;             // the first workgroup of this plane on that XCD
    w.step = (nx - 1 - xfirst) / 8 + 1;
    w.first = (int)((long long)n_tiles * xcd / 8) + (x - xfirst) / 8;
    w.end = (int)((long long)n_tiles * (xcd + 1) / 8);
    return w;
}

// ---- pieces shared by the kernels that hold their input window in LDS ----------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// Loads that must not wait for asynchronous LDS loads in flight are made through pointers that
// name global memory: a generic pointer could point into LDS and the compiler would drain every
// outstanding LDS write first.
#define ENS_GLOBAL(T, p) ((const __attribute__((address_space(1))) T*)(p))
// Stores likewise: a store through a generic pointer is a flat instruction, which also counts as
// an LDS operation, so the next LDS read would wait for the store to leave the wave.
#define ENS_GLOBAL_W(T, p) ((__attribute__((address_space(1))) T*)(p))

// Pixels in a padded raster: image n, row hi, column wi sits at position (n * H1 + hi) * W1 + wi
// with H1 >= H, W1 >= W; the positions with hi >= H or wi >= W hold no pixel.  Fills
// tbl[q] for q in [0, rows) with the pixel index (n * H + hi) * W + wi of position first + q,
// or -1 for positions without a pixel or outside [0, PP).  All threads of the workgroup call it.
__device__ __forceinline__ void raster_table(int* tbl, int rows, int first, int PP, int H1, int W1, int H, int W) {
    const int img = H1 * W1;
    const float inv_img = __builtin_amdgcn_rcpf((float)img), inv_w1 = __builtin_amdgcn_rcpf((float)W1);
    for (int q = threadIdx.x; q < rows; q += blockDim.x) {
        const int pp = first + q;
        int p = -1;
        if (pp >= 0 && pp < PP) {
            // the float quotients are off by one at most (pp < 2^24): one correction step each
            int n = (int)((float)pp * inv_img);
            int rem = pp - n * img;
            n += (rem >= img ? 1 : 0) - (rem < 0 ? 1 : 0);
            rem = pp - n * img;
            int hi = (int)((float)rem * inv_w1);
            int wi = rem - hi * W1;
            hi += (wi >= W1 ? 1 : 0) - (wi < 0 ? 1 : 0);
            wi = rem - hi * W1;
            if (hi < H && wi < W) p = (n * H + hi) * W + wi;
        }
        tbl[q] = p;
    }
}

// What the epilogue of a BP x BC tile needs from memory, asked for before the main loop: scale and
// bias of this thread's 8 channels and the residual values of its BP * BC / 2048 output groups.
template <int BP, int BC>
struct TilePrefetch {
    static constexpr int G = BC / 8;                 // 8-channel groups per output row
    static constexpr int RPI = 256 / G;              // output rows the workgroup stores per pass
    static constexpr int NI = BP / RPI;              // 16-byte output groups per thread
    f32x4 bias0, bias1, scale0, scale1;
    u32x4 res[NI];
    int co;                                          // first of this thread's 8 channels
    bool cok, has_res;
    // own: this tile's output rows in the table (own[r] = pixel of output row r, -1: none)
    __device__ __forceinline__ void load(const ConvArgs& a, const int* own, int c0, bool partial) {
        const int t = threadIdx.x;
        co = c0 + (t % G) * 8;
        cok = co < a.cout;
        bias0 = f32x4{0.f, 0.f, 0.f, 0.f};
        bias1 = bias0;
        scale0 = f32x4{1.f, 1.f, 1.f, 1.f};
        scale1 = scale0;
        if (cok && !partial) {
            bias0 = *ENS_GLOBAL(f32x4, a.bias + co);
            bias1 = *ENS_GLOBAL(f32x4, a.bias + co + 4);
            scale0 = *ENS_GLOBAL(f32x4, a.scale + co);
            scale1 = *ENS_GLOBAL(f32x4, a.scale + co + 4);
        }
        const uint16_t* rg = partial ? nullptr : (const uint16_t*)a.res.p;
        has_res = rg != nullptr;
#pragma unroll
        for (int i = 0; i < NI; i++) res[i] = u32x4{0u, 0u, 0u, 0u};
        if (rg) {
#pragma unroll
            for (int i = 0; i < NI; i++) {
                const int p = own[t / G + RPI * i];
                if (p >= 0 && cok) res[i] = *ENS_GLOBAL(u32x4, rg + (size_t)p * a.res.stride + a.res.c0 + co);
            }
        }
    }
};

// Epilogue of a BP x BC tile held in the accumulators of 4 waves (wave tile TP x TC blocks of
// 32 x 32 at rows wp0, channels wc0): the tile is turned round in LDS (fp32, HROWS rows at a time,
// rows padded by 16 bytes) and leaves as 16-byte groups of 8 channels with scale, bias, residual
// and activation applied, or, when `partial` (a share of the K range), as fp32 sums into slice
// `slice` of the workspace.  Rows whose table entry is negative are dropped.  The caller has
// made sure that nobody still uses the LDS behind otile.
template <int BP, int BC, int TP, int TC, int HROWS>
__device__ __forceinline__ void store_tile(const ConvArgs& a, f32x16 (&acc)[TC][TP], float* otile, const int* own,
                                           const TilePrefetch<BP, BC>& pf, int wp0, int wc0, bool partial, int slice,
                                           int P) {
    constexpr int OROW = BC + 4, G = BC / 8, RPI = 256 / G;
    static_assert(256 % G == 0 && HROWS % RPI == 0 && BP % HROWS == 0, "a thread keeps its channel group over the passes");
    const int t = threadIdx.x, lane = t & 63, lrow = lane & 31, lhalf = lane >> 5;
    const int g8 = t % G, rbase = t / G;
    uint16_t* __restrict__ yg = (uint16_t*)a.y.p;
#pragma unroll
    for (int h0 = 0; h0 < BP; h0 += HROWS) {
        if (h0 > 0) __syncthreads();
#pragma unroll
        for (int j = 0; j < TP; j++) {
            const int rb = wp0 + j * 32;
            if (rb < h0 || rb >= h0 + HROWS) continue;
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int g = 0; g < 4; g++)
                    *(float4*)&otile[(rb - h0 + lrow) * OROW + wc0 + i * 32 + g * 8 + lhalf * 4] =
                        make_float4(acc[i][j][g * 4], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]);
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < HROWS / RPI; it++) {
            const int row = rbase + RPI * it;                    // within this chunk
            const int item = h0 / RPI + it;                      // among this thread's groups
            const int p = own[h0 + row];
            if (p < 0 || !pf.cok) continue;
            const float4 lo = *(const float4*)&otile[row * OROW + g8 * 8];
            const float4 hi = *(const float4*)&otile[row * OROW + g8 * 8 + 4];
            if (partial) {
                float* d = a.ws + ((size_t)slice * (size_t)P + (size_t)p) * a.cout + pf.co;
                *ENS_GLOBAL_W(f32x4, d) = f32x4{lo.x, lo.y, lo.z, lo.w};
                *ENS_GLOBAL_W(f32x4, d + 4) = f32x4{hi.x, hi.y, hi.z, hi.w};
                continue;
            }
            float v[8] = {fmaf(lo.x, pf.scale0.x, pf.bias0.x), fmaf(lo.y, pf.scale0.y, pf.bias0.y),
                          fmaf(lo.z, pf.scale0.z, pf.bias0.z), fmaf(lo.w, pf.scale0.w, pf.bias0.w),
                          fmaf(hi.x, pf.scale1.x, pf.bias1.x), fmaf(hi.y, pf.scale1.y, pf.bias1.y),
                          fmaf(hi.z, pf.scale1.z, pf.bias1.z), fmaf(hi.w, pf.scale1.w, pf.bias1.w)};
            if (pf.has_res) {
                const uint32_t rr[4] = {pf.res[item].x, pf.res[item].y, pf.res[item].z, pf.res[item].w};
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    v[2 * q] += bf16_to_f32((uint16_t)(rr[q] & 0xFFFF));
                    v[2 * q + 1] += bf16_to_f32((uint16_t)(rr[q] >> 16));
                }
            }
            apply_act_n<8>(v, a.act);
            uint32_t o[4];
#pragma unroll
            for (int q = 0; q < 4; q++) o[q] = pack_bf16x2(v[2 * q], v[2 * q + 1]);
            *ENS_GLOBAL_W(u32x4, yg + (size_t)p * a.y.stride + a.y.c0 + pf.co) = u32x4{o[0], o[1], o[2], o[3]};
        }
    }
}

// Stride-1 convolution over a 16-channel input with filter and window resident in LDS (the input
// stems after the space-to-depth rewrite); defined in conv_taps.hip.
bool conv_taps_applicable(const ConvArgs& a, int nb);
const char* conv_taps_name(const ConvArgs& a);
hipError_t launch_conv_taps(const ConvArgs& a, const ConvArgs* argv, int G, int nb, hipStream_t s);

// The input stem and the 3x3 / stride-2 max-pool behind it as one kernel; defined in conv_stempool.hip.
// `pool` carries the pooled output (y, Ho, Wo); argv: G blocks of the convolution, then G of the pool.
bool conv_stempool_applicable(const ConvArgs& a, const ConvArgs& pool, int nb, int G);
const char* conv_stempool_name();
hipError_t launch_conv_stempool(const ConvArgs& a, const ConvArgs& pool, const ConvArgs* argv, int G, int nb, hipStream_t s);

// Register-staged variant (pre-activated inputs); defined in conv_regstage.hip.
hipError_t launch_conv_regstage(const ConvArgs& a, const ConvArgs* argv, int G, int nb, int P, hipStream_t s);
const char* conv_regstage_name(const ConvArgs& a, int P);

// Second pass of a convolution whose K range was split: sums the `splits` fp32 slices of P x cout
// partial sums in the workspace and applies bias, residual and activation; defined in conv_mfma.hip.
hipError_t launch_conv_splitk_epilogue(const ConvArgs& a, const ConvArgs* argv, int G, int nb, int P, int splits, hipStream_t s);

// 3x3 stride-1 kernel with the filter in registers and persistent workgroups; defined in conv_wreg.hip.
bool conv_wreg_applicable(const ConvArgs& a, int nb, int G);
const char* conv_wreg_name(const ConvArgs& a);
hipError_t launch_conv_wreg(const ConvArgs& a, const ConvArgs* argv, int G, int nb, hipStream_t s);

// A residual bottleneck (1x1, 3x3, 1x1 with the residual) as one kernel, the two tensors in between
// held in LDS; defined in conv_bneck.hip.  argv: G blocks of the first convolution, then G of the
// second, then G of the third.
bool conv_bneck_applicable(const ConvArgs& a1, const ConvArgs& a2, const ConvArgs& a3, int nb, int G);
const char* conv_bneck_name(const ConvArgs& a1);
hipError_t launch_conv_bneck(const ConvArgs& a1, const ConvArgs& a2, const ConvArgs& a3, const ConvArgs* argv, int G, int nb,
                             hipStream_t s);

// 1x1 stride-1 kernel that takes its weights straight from memory in matrix-core operand order (a.wpk);
// defined in conv_pw.hip.
bool conv_pw_applicable(const ConvArgs& a, int nb, int G);
const char* conv_pw_name(const ConvArgs& a, int G);
hipError_t launch_conv_pw(const ConvArgs& a, const ConvArgs* argv, int G, int nb, hipStream_t s);

// 3x3 stride-1 kernel with the input window resident in LDS; defined in conv_halo.hip.
// conv_halo_pick returns the variant that runs the layer, or -1 when the generic kernel does.
int conv_halo_pick(const ConvArgs& a, int nb, int G);
const char* conv_halo_name(int variant);
hipError_t launch_conv_halo(const ConvArgs& a, const ConvArgs* argv, int G, int nb, int variant, hipStream_t s);

}  // namespace ens
