// Input stem and the max-pool behind it as one kernel: a 4x4-tap stride-1 convolution over the
// 16-channel space-to-depth image (the 7x7 / stride-2 stem of the residual and dense networks after
// its rewrite, see conv_taps.hip) with ReLU, followed by a 3x3 / stride-2 / padding-1 max-pool.
//
// Run as two kernels the stem writes 64 channels of every one of its output pixels and the pool reads
// them straight back (147 MiB each way for 96 images of 224 x 224); here only the pooled map, a
// quarter of that, leaves the chip.  A workgroup works on a band of one image: the 2*KB + 1 rows of
// stem output that KB rows of pooled output need (neighbouring bands share one row, which is
// computed twice).  In the padded raster of the stem kernel those rows are one run of consecutive
// positions, cut into sub-tiles of 128 positions that go through the resident-filter matrix-core loop
// of the stem kernel one after the other (next window arriving meanwhile); their outputs (scale,
// bias, ReLU, bf16) go to a tile in LDS, zeros at positions that hold no pixel, and after the last
// sub-tile the workgroup takes the 3x3 maxima from there.  Zeros stand in for the pool's padding:
// after a ReLU no value is below zero and every window holds at least one pixel.
//
// LDS rows of the tile are 128 bytes (64 channels, half of the 64 banks); the 16-byte chunks of row q are
// swizzled by (q / 2) mod 8 to spread a wavefront's stores (one row per lane) and the pool's loads over the banks.
#include "conv_common.h"

#include <type_traits>
#include <utility>

namespace ens {

typedef __attribute__((address_space(3))) void* lds_ptr_t;

template <int OFFSET>
__device__ __forceinline__ bf16x8 sp_lds_read(uint32_t addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
    return v;
}

template <class F, int... T>
__device__ __forceinline__ void sp_for_each(F&& f, std::integer_sequence<int, T...>) {
    (f(std::integral_constant<int, T>{}), ...);
}

constexpr int SP_BP = 128;        // positions per sub-tile
constexpr int SP_KB = 2;          // pooled rows per band
constexpr int SP_BROWS = 2 * SP_KB + 1;

// argv: G blocks of the convolution, then G blocks that describe the pooled output (y, Ho, Wo)
template <int KH, int KW>
__global__ __launch_bounds__(256) void stem_pool_bf16(const ConvArgs* __restrict__ argv, const int nb_, const int hrows,
                                                      const int gh, const int gw, const int nsub) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const ConvArgs a = argv[blockIdx.z];
    const ConvArgs pool = argv[gridDim.z + blockIdx.z];
    constexpr int BP = SP_BP, BC = 64, NT = KH * KW, TC = 2;

    const int W1 = a.W + gw, H1 = a.H + gh;
    const int PP = nb_ * H1 * W1;
    const int PH = pool.Ho, PW = pool.Wo;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wp0 = wave * 32;
    const int c0 = blockIdx.y * BC;
    const int hbytes = hrows * 32, nhl = hrows / 128;            // bytes and load instructions per band window
    const int orows = nsub * BP;                                 // positions a band is computed for
    const int phb = (PH + SP_KB - 1) / SP_KB;                    // bands per image
    const int n_bands = nb_ * phb;

    // LDS: window 0 | window 1 | window tables 0, 1 | output tables 0, 1 | the band's stem output
    int* const tbls = (int*)(lds + 2 * hbytes);      // window row -> input pixel index, -1: no pixel
    int* const owns = tbls + 2 * hrows;              // position of the band -> output pixel index, -1: none
    unsigned char* const ctile = (unsigned char*)(owns + 2 * orows);
    const int origin = a.pt * W1 + a.pl;             // window row 0 is tap (0, 0) of the band's first position

    constexpr unsigned OOBV = 0x80000000u;           // past the end of every buffer the launcher admits: zeros (loads), dropped (stores)
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.x.p, 0, (int)((unsigned)nb_ * (unsigned)(a.H * a.W) * (unsigned)a.x.stride * 2u), 0x00020000);
    const int r0 = t >> 1;                                       // window row k * 128 + r0, half t & 1
    const unsigned xlane = (unsigned)(a.x.c0 * 2 + (((t & 1) ^ ((r0 >> 3) & 1)) * 16));
    // first raster position of band b: one stem row above the centre row of its first pooled row
    auto band_start = [&](int b) {
        const int n = b / phb, jb = b - n * phb;
        return (n * H1 + 2 * SP_KB * jb - 1) * W1;
    };
    auto make_tables = [&](int buf, int start) {
        raster_table(tbls + buf * hrows, hrows, start - origin, PP, H1, W1, a.H, a.W);
        raster_table(owns + buf * orows, orows, start, PP, H1, W1, a.Ho, a.Wo);
    };
    auto issue_window = [&](int buf) {
        const int* tbl = tbls + buf * hrows;
        unsigned char* dst = lds + buf * hbytes + wave * 1024;
        for (int k0 = 0; k0 < nhl; k0 += 4) {
            int p4[4];
#pragma unroll
            for (int j = 0; j < 4; j++) p4[j] = tbl[min(k0 + j, nhl - 1) * 128 + r0];
#pragma unroll
            for (int j = 0; j < 4; j++) {
                if (k0 + j >= nhl) break;
                const unsigned vo = p4[j] >= 0 ? (unsigned)(p4[j] * a.x.stride * 2) + xlane : OOBV;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (lds_ptr_t)(dst + (k0 + j) * 4096), LDS_LOAD_BYTES, vo, 0, 0, 0);
            }
        }
    };
    const TileWalk walk = tile_walk(n_bands, (blockIdx.y + blockIdx.z * gridDim.y) * gridDim.x);
    int band = walk.first;
    if (band >= walk.end) return;
    make_tables(0, band_start(band));
    __syncthreads();
    issue_window(0);

    // ---- the filter stays in registers for the workgroup's whole life: fragment (tap, i) of this lane is
    //      half lane / 32 of weight row 32 i + r', r' = lane % 32 with bits 2 and 3 swapped (a lane's 16
    //      results of a block are then two runs of 8 consecutive channels); weights are [cout][tap][16]
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int prow = (lrow & 0x13) | ((lrow & 4) << 1) | ((lrow & 8) >> 1);
    bf16x8 wreg[NT][TC];
    {
        const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
            (void*)a.w, 0, (int)((unsigned)a.cout * (unsigned)(NT * 16) * 2u), 0x00020000);
#pragma unroll
        for (int i = 0; i < TC; i++) {
            const int co = c0 + 32 * i + prow;
            const unsigned base = co < a.cout ? (unsigned)(co * NT * 32 + lhalf * 16) : OOBV;
#pragma unroll
            for (int tap = 0; tap < NT; tap++)
                wreg[tap][i] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(wres, base, tap * 32, 0));
        }
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
    const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)pool.y.p, 0, (int)((unsigned)nb_ * (unsigned)(PH * PW) * (unsigned)pool.y.stride * 2u), 0x00020000);

    // scale and bias of this lane's 4 runs of 8 channels (32 i + 16 k + 8 (lane / 32) + 0..7) stay in registers:
    // with one wavefront per SIMD there are registers to spare and no second wavefront to hide an LDS round trip
    f32x4 sq[TC][2][2], bq[TC][2][2];
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int k = 0; k < 2; k++) {
            const int cb = 32 * i + 16 * k + 8 * lhalf;
            const bool ok = c0 + cb < a.cout;                    // channel counts come in 8s: a run exists or does not
#pragma unroll
            for (int h = 0; h < 2; h++) {
                sq[i][k][h] = ok ? *ENS_GLOBAL(f32x4, a.scale + c0 + cb + 4 * h) : f32x4{1.f, 1.f, 1.f, 1.f};
                bq[i][k][h] = ok ? *ENS_GLOBAL(f32x4, a.bias + c0 + cb + 4 * h) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
    // the maxima: task idx = t + 256 j is (pooled row idx / 8 / PW of the band, pooled column idx / 8 % PW, channels
    // 8 (idx % 8) ..); what does not depend on the band is worked out once
    constexpr int NTASK = (SP_KB * 128 * 8 + 255) / 256;         // pooled rows of up to 128 columns
    int task_q[NTASK], task_y[NTASK];                            // tile row of the window's top-left corner; output offset less the band's
    bool task_ok[NTASK];
    int task_jr[NTASK];                                          // pooled row of the band
    bool task_left[NTASK];                                       // the window's first column lies left of the image
#pragma unroll
    for (int j = 0; j < NTASK; j++) {
        const int idx = t + 256 * j;
        const int g = idx & 7, pc = (idx >> 3) % PW, jr = (idx >> 3) / PW;
        const bool ok = jr < SP_KB && c0 + 8 * g < a.cout;
        task_ok[j] = ok;
        task_q[j] = (2 * jr) * W1 + 2 * pc - 1;
        task_left[j] = pc == 0;
        task_jr[j] = jr;
        task_y[j] = ((jr * PW + pc) * pool.y.stride + pool.y.c0 + c0 + 8 * g) * 2;
    }

    // Per band: its window has landed; ask for the next band's (tables first); run the sub-tiles, each wave on
    // its own 32 positions of every sub-tile with no barrier in between; then the maxima.
    for (int buf = 0; band < walk.end; band += walk.step, buf ^= 1) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // this band's window (and, the first time, the filter): this wave's part,
        __syncthreads();                                         // everybody's; the previous band's maxima have been taken from the tile
        const bool has_next = band + walk.step < walk.end;
        if (has_next) {
            make_tables(buf ^ 1, band_start(band + walk.step));
            __syncthreads();                                     // tables written; the other window was free since the barrier above
            issue_window(buf ^ 1);
        }
        const uint32_t halo0 = lds0 + (uint32_t)(buf * hbytes);
        // Pixel fragments come through a ring of four registers, three taps ahead of their use (LDS returns in
        // order: tap t is complete once no more than the reads issued after it are outstanding).  The ring does
        // not live across sub-tiles: a value asked for by hand must not be moved by the compiler while in flight.
        bf16x8 xf[4];
        auto issue_frag = [&](int sub, auto tap_c) {
            constexpr int tap = decltype(tap_c)::value;
            const uint32_t q = (uint32_t)(sub * BP + wp0 + lrow + (tap / KW) * W1 + tap % KW);
            xf[tap & 3] = sp_lds_read<0>(halo0 + q * 32 + ((((uint32_t)lhalf) ^ ((q >> 3) & 1)) << 4));
        };
        auto issue_first = [&](int sub) {
            issue_frag(sub, std::integral_constant<int, 0>{});
            issue_frag(sub, std::integral_constant<int, 1>{});
            issue_frag(sub, std::integral_constant<int, 2>{});
            issue_frag(sub, std::integral_constant<int, 3>{});
        };
        auto run_sub = [&](int sub) {
            const int q0 = sub * BP + wp0 + lrow;                // this lane's position of the band
            issue_first(sub);
            f32x16 acc[TC];
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int v = 0; v < 16; v++) acc[i][v] = 0.f;
            sp_for_each([&](auto tap_c) {
                constexpr int tap = decltype(tap_c)::value;
                constexpr int ahead = NT - 1 - tap < 3 ? NT - 1 - tap : 3;
                asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(xf[tap & 3]) : "n"(ahead));
#pragma unroll
                for (int i = 0; i < TC; i++) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[tap][i], xf[tap & 3], acc[i], 0, 0, 0);
                if constexpr (tap + 4 < NT) issue_frag(sub, std::integral_constant<int, (tap + 4 < NT ? tap + 4 : tap)>{});
            }, std::make_integer_sequence<int, NT>{});
            const int pout = owns[buf * orows + q0];
            // ---- this sub-tile's stem output into the band's tile: register v of a lane is channel
            //      32i + 16(v/8) + 8(lane/32) + v%8 of its position; scale, bias, ReLU, bf16
            unsigned char* const row = ctile + q0 * 128;
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int k = 0; k < 2; k++) {
                    uint32_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        const float v0 = fmaf(acc[i][8 * k + 2 * e], sq[i][k][e >> 1][(2 * e) & 3], bq[i][k][e >> 1][(2 * e) & 3]);
                        const float v1 = fmaf(acc[i][8 * k + 2 * e + 1], sq[i][k][e >> 1][(2 * e + 1) & 3], bq[i][k][e >> 1][(2 * e + 1) & 3]);
                        // ReLU on the rounded pair: a negative bf16 is a negative 16-bit integer
                        typedef short s16x2 __attribute__((ext_vector_type(2)));
                        const s16x2 z = {0, 0};
                        o[e] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, pack_bf16x2(v0, v1)), z));
                    }
                    const u32x4 val = pout >= 0 ? u32x4{o[0], o[1], o[2], o[3]} : u32x4{0u, 0u, 0u, 0u};
                    *(u32x4*)(row + ((((4 * i + 2 * k + lhalf) ^ ((q0 >> 1) & 7))) << 4)) = val;
                }
        };
        for (int sub = 0; sub < nsub; sub++) run_sub(sub);
        __syncthreads();                                         // the band's tile is complete
        // ---- 3x3 / stride-2 maxima; to the right of an image lies a gap column, below it a gap row: zeros in the tile
        const int n = band / phb, jb = band - n * phb;
        const int j0 = SP_KB * jb;
        const unsigned yband = (unsigned)((n * PH + j0) * PW) * (unsigned)pool.y.stride * 2u;
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        s16x8 mx[NTASK];
#pragma unroll
        for (int j = 0; j < NTASK; j++) {
            mx[j] = s16x8{0, 0, 0, 0, 0, 0, 0, 0};
            if (!task_ok[j]) continue;
            const int g = (t + 256 * j) & 7;
            // neighbouring groups of 8 lanes read columns two apart: rows of the same bank half.  Every other
            // group takes the three columns of its window in rotated order, so that the two never meet.
            const int rot = ((t + 256 * j) >> 3) & 1;
#pragma unroll
            for (int dr = 0; dr < 3; dr++)
#pragma unroll
                for (int d3 = 0; d3 < 3; d3++) {
                    const int dc = d3 + rot >= 3 ? d3 + rot - 3 : d3 + rot;
                    if (dc == 0 && task_left[j]) continue;       // left of the image: padding
                    const int q = task_q[j] + dr * W1 + dc;
                    const s16x8 v = *(const s16x8*)(ctile + q * 128 + ((g ^ ((q >> 1) & 7)) << 4));
                    mx[j] = __builtin_elementwise_max(mx[j], v); // non-negative bf16 values order like 16-bit integers
                }
        }
#pragma unroll
        for (int j = 0; j < NTASK; j++) {
            const unsigned yo = task_ok[j] && j0 + task_jr[j] < PH ? yband + (unsigned)task_y[j] : OOBV;
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, mx[j]), yres, yo, 0, 0);
        }
    }
}

// ---- host side -----------------------------------------------------------------------------
constexpr int SP_LDS_LIMIT = 160 * 1024;
constexpr int SP_CUS = 256;

struct StemPoolPlan { int hrows, gh, gw, nsub, wgs; size_t bytes; };

// conv: the stem after its space-to-depth rewrite (16 stored input channels, 4x4 taps, stride 1, ReLU, no
// residual); pool: its output size, the result of a 3x3 / stride-2 / padding-1 max-pool over the stem's output
static bool stempool_plan(const ConvArgs& a, const ConvArgs& pool, int nb, int G, StemPoolPlan* pl) {
    if (a.cin != 16 || a.sh != 1 || a.sw != 1 || a.pre_scale || a.res.p || a.cout % 8 || a.act != ACT_RELU) return false;
    if (a.kh != 4 || a.kw != 4 || a.Ho > a.H || a.Wo > a.W) return false;
    if (pool.Ho != (a.Ho - 1) / 2 + 1 || pool.Wo != (a.Wo - 1) / 2 + 1) return false;
    const int pb = a.Ho - 1 + a.kh - a.pt - a.H, pr = a.Wo - 1 + a.kw - a.pl - a.W;   // bottom / right padding
    pl->gh = a.pt > pb ? a.pt : (pb > 0 ? pb : 0);
    pl->gw = a.pl > pr ? a.pl : (pr > 0 ? pr : 0);
    if (pl->gh < 1) pl->gh = 1;                       // the row above an image's first must hold no pixel
    if (pl->gw < 1) pl->gw = 1;                       // and so must the column right of its last
    if ((long long)nb * a.H * a.W * a.x.stride * 2 >= 0x7FFFFF00LL) return false;
    if ((long long)nb * pool.Ho * pool.Wo * pool.y.stride * 2 >= 0x7FFFFF00LL) return false;
    const int W1 = a.W + pl->gw;
    const long long PP = (long long)nb * (a.H + pl->gh) * W1;
    if (PP >= (1LL << 24)) return false;
    pl->nsub = (SP_BROWS * W1 + SP_BP - 1) / SP_BP;
    const int orows = pl->nsub * SP_BP;
    const int need = orows + (a.kh - 1) * W1 + a.kw;             // window of a whole band
    pl->hrows = (need + 127) / 128 * 128;
    pl->bytes = 2 * ((size_t)pl->hrows * 32 + (size_t)pl->hrows * 4 + (size_t)orows * 4) + (size_t)orows * 128;
    if (pool.Wo > 128) return false;                  // the maxima of a band are dealt to the threads once, for up to 128 columns
    if (pl->bytes > (size_t)SP_LDS_LIMIT) return false;
    // as many workgroups as the chip holds at once, shared by the gang and the channel tiles, and not one more
    const int per_cu = (int)((size_t)SP_LDS_LIMIT / pl->bytes) < 1 ? 1 : (int)((size_t)SP_LDS_LIMIT / pl->bytes);
    const int ctiles = (a.cout + 63) / 64;
    long long wgs = ((long long)SP_CUS * per_cu) / ((long long)G * ctiles);
    if (wgs < 1) wgs = 1;
    const long long bands = (long long)nb * ((pool.Ho + SP_KB - 1) / SP_KB);
    pl->wgs = (int)(wgs < bands ? wgs : bands);
    return true;
}

bool conv_stempool_applicable(const ConvArgs& a, const ConvArgs& pool, int nb, int G) {
    StemPoolPlan pl;
    return stempool_plan(a, pool, nb, G, &pl);
}

const char* conv_stempool_name() { return "stem_pool_bf16<4x4>"; }

hipError_t launch_conv_stempool(const ConvArgs& a, const ConvArgs& pool, const ConvArgs* argv, int G, int nb, hipStream_t s) {
    StemPoolPlan pl;
    if (!stempool_plan(a, pool, nb, G, &pl)) return hipErrorInvalidValue;
    if (a.x.stride % 8 || a.x.c0 % 8 || pool.y.stride % 8 || pool.y.c0 % 8) return hipErrorInvalidValue;
    static bool raised = false;                                  // LDS above 64 KB has to be asked for once
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void*)&stem_pool_bf16<4, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, SP_LDS_LIMIT);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const dim3 grid((unsigned)pl.wgs, (unsigned)((a.cout + 63) / 64), G);
    ENS_LAUNCH((stem_pool_bf16<4, 4>), grid, dim3(256), pl.bytes, s, argv, nb, pl.hrows, pl.gh, pl.gw, pl.nsub);
    return hipGetLastError();
}

}  // namespace ens
