// Stride-1 convolution over a 16-channel input (the image stored space-to-depth: the input
// stems) on the CDNA4 matrix cores, with everything a workgroup reads resident in LDS.
//
// One filter tap of 16 channels is exactly the K = 16 of v_mfma_f32_32x32x16_bf16, and the whole
// filter of a 64-channel output tile (KH*KW taps x 64 x 32 bytes, 32 KB for 4x4) fits LDS next
// to the input window.  A workgroup therefore loads its weights and its window once, waits
// once, and then runs KH*KW matrix-core steps per accumulator without another barrier or load.
//
// Pixels are numbered in a padded raster (see conv_halo.hip): row length W + gw and H + gh rows
// per image, where the gaps gw = max(left, right padding) and gh = max(top, bottom padding) hold
// no pixel and are loaded as zeros, so tap (kh, kw) of any output position lies
// (kh - pt) * (W + gw) + (kw - pl) positions further on.  A workgroup of 4 wavefronts owns BP
// consecutive positions x 64 output channels; each wavefront BP/4 positions x 64 channels.
//
// LDS rows are 32 bytes (one position or one output channel of one tap); the two 16-byte halves
// of row r are swapped when bit 3 of r is set, so that the 16 rows a quarter-wavefront reads
// cover all 64 banks.
#include "conv_common.h"

#include <type_traits>
#include <utility>

namespace ens {

typedef __attribute__((address_space(3))) void* lds_ptr_t;

template <int OFFSET>
__device__ __forceinline__ bf16x8 taps_lds_read(uint32_t addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
    return v;
}

template <class F, int... T>
__device__ __forceinline__ void for_each_tap(F&& f, std::integer_sequence<int, T...>) {
    (f(std::integral_constant<int, T>{}), ...);
}

// The workgroups of one (member, channel tile) are persistent: each takes a share of the position
// tiles (tile_walk: neighbouring tiles on one XCD).  The filter is loaded once; the window of the next tile arrives in a
// second buffer while the matrix cores work on the current one and while its output leaves
// straight from the accumulators: the filter rows go to the matrix cores with bits 2 and 3 of the row
// number swapped, which makes a lane's 16 results of a 32x32 block two runs of 8 consecutive channels
// (two 16-byte stores) after the per-channel scale and bias.
template <int BP, int KH, int KW>
__global__ __launch_bounds__(256) void conv_taps16_bf16(const ConvArgs* __restrict__ argv, const int nb_,
                                                        const int hrows, const int gh, const int gw) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const ConvArgs a = argv[blockIdx.z];
    constexpr int BC = 64, NT = KH * KW;
    constexpr int WTP = BP / 4;                      // positions per wave, all 64 channels
    constexpr int TP = WTP / 32, TC = 2;
    static_assert(TP == 1 || TP == 2, "32 or 64 positions per wave");
    constexpr int WBYTES = NT * BC * 32;             // the resident filter
    static_assert(WBYTES % 4096 == 0, "whole load instructions");

    const int W1 = a.W + gw, H1 = a.H + gh;
    const int PP = nb_ * H1 * W1;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wp0 = wave * WTP;
    const int n_ptiles = (PP + BP - 1) / BP;
    const int c0 = blockIdx.y * BC;
    const int hbytes = hrows * 32, nhl = hrows / 128;            // bytes and load instructions per window

    // LDS: filter | window 0 | window 1 | window tables 0, 1 | output tables 0, 1 | bias, then scale, of the 64 channels
    unsigned char* const halo = lds + WBYTES;
    int* const tbls = (int*)(halo + 2 * hbytes);     // window row -> input pixel index, -1: no pixel
    int* const owns = tbls + 2 * hrows;              // position of the tile -> output pixel index, -1: none
    float* const biasl = (float*)(owns + 2 * BP);
    float* const scalel = biasl + BC;
    const int origin = a.pt * W1 + a.pl;             // window row 0 is tap (0, 0) of the tile's first position

    // ---- loads.  Offsets past the end of a buffer give zeros in LDS; 2^31 is past the end of
    //      every buffer the launcher admits.
    constexpr unsigned OOBV = 0x80000000u;
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.x.p, 0, (int)((unsigned)nb_ * (unsigned)(a.H * a.W) * (unsigned)a.x.stride * 2u), 0x00020000);
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.w, 0, (int)((unsigned)a.cout * (unsigned)(NT * 16) * 2u), 0x00020000);
    {
        // LDS position k * 4096 + t * 16 is half (t & 1) of channel row (t & 127) / 2 of tap
        // 2k + t / 128; the weights are [cout][tap][16] in memory
        const int co = (t & 127) >> 1, half = (t & 1) ^ ((co >> 3) & 1);
        const unsigned base = c0 + co < a.cout ? (unsigned)((c0 + co) * NT * 32 + (t >> 7) * 32 + half * 16) : OOBV;
#pragma unroll
        for (int k = 0; k < WBYTES / 4096; k++)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wres, (lds_ptr_t)(lds + k * 4096 + wave * 1024), LDS_LOAD_BYTES, base, k * 64, 0, 0);
    }
    const int r0 = t >> 1;                                       // window row k * 128 + r0, half t & 1
    const unsigned xlane = (unsigned)(a.x.c0 * 2 + (((t & 1) ^ ((r0 >> 3) & 1)) * 16));
    auto make_tables = [&](int buf, int ptile) {
        raster_table(tbls + buf * hrows, hrows, ptile * BP - origin, PP, H1, W1, a.H, a.W);
        raster_table(owns + buf * BP, BP, ptile * BP, PP, H1, W1, a.Ho, a.Wo);
    };
    auto issue_window = [&](int buf) {
        const int* tbl = tbls + buf * hrows;
        unsigned char* dst = halo + buf * hbytes + wave * 1024;
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
    const TileWalk walk = tile_walk(n_ptiles, (blockIdx.y + blockIdx.z * gridDim.y) * gridDim.x);
    int ptile = walk.first;
    if (ptile >= walk.end) {                                     // nothing to do: let the filter loads land and leave
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }
    make_tables(0, ptile);
    if (t < BC) {
        biasl[t] = c0 + t < a.cout ? a.bias[c0 + t] : 0.f;
        scalel[t] = c0 + t < a.cout ? a.scale[c0 + t] : 1.f;
    }
    __syncthreads();
    issue_window(0);

    // ---- fragment side: lane reads row (lane & 31) of each 32-row block, half lane / 32; of the
    //      filter the row with bits 2 and 3 swapped
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int prow = (lrow & 0x13) | ((lrow & 4) << 1) | ((lrow & 8) >> 1);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
    const uint32_t wa = lds0 + (uint32_t)(prow * 32 + ((lhalf ^ ((prow >> 3) & 1)) << 4));
    const uint32_t lq = (uint32_t)(wp0 + lrow);
    // this lane's output channels: cl + 32i + 16k + 0..7; out-of-range offsets drop a store
    constexpr unsigned OOBS = 0x80000000u;
    const int cl = c0 + 8 * lhalf;
    const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.y.p, 0, (int)((unsigned)nb_ * (unsigned)(a.Ho * a.Wo) * (unsigned)a.y.stride * 2u), 0x00020000);

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");             // filter and first window have landed: this wave's part,
    __builtin_amdgcn_s_barrier();                                // and with the barrier everybody's

    // Per tile: ask for the next window, compute, wait for the next window, send the output off.
    // The one wait counter covers loads and stores alike, so the wait sits before this tile's
    // stores are issued: by then the previous tile's stores have had a whole compute phase to
    // complete and do not hold it up.
    for (int buf = 0; ptile < walk.end; ptile += walk.step, buf ^= 1) {
        const bool has_next = ptile + walk.step < walk.end;
        if (has_next) {
            make_tables(buf ^ 1, ptile + walk.step);
            __syncthreads();                                     // tables written; the other buffer is free (see the end of the loop)
            issue_window(buf ^ 1);
        }

        // this tile's output pixels are read before the barrier below: the table is rewritten after it
        int pout[TP];
#pragma unroll
        for (int j = 0; j < TP; j++) pout[j] = owns[buf * BP + wp0 + lrow + 32 * j];
        f32x16 acc[TC][TP];
#pragma unroll
        for (int i = 0; i < TC; i++)
#pragma unroll
            for (int j = 0; j < TP; j++)
#pragma unroll
                for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;
        const uint32_t halo0 = lds0 + WBYTES + (uint32_t)(buf * hbytes);
        bf16x8 wf[2][TC], xf[2][TP];
        auto read_frags = [&](auto tap_c, int b) {
            constexpr int tap = decltype(tap_c)::value;
            const uint32_t q = lq + (uint32_t)((tap / KW) * W1 + tap % KW);
            const uint32_t xa = halo0 + q * 32 + ((((uint32_t)lhalf) ^ ((q >> 3) & 1)) << 4);
            wf[b][0] = taps_lds_read<tap * 2048>(wa);
            wf[b][1] = taps_lds_read<tap * 2048 + 1024>(wa);
            xf[b][0] = taps_lds_read<0>(xa);
            if (TP > 1) xf[b][1 % TP] = taps_lds_read<1024>(xa);
        };
        auto step = [&](auto tap_c) {
            constexpr int tap = decltype(tap_c)::value;
            constexpr int b = tap & 1;
            // the next tap's reads are issued first; LDS returns in order, so once no more than
            // those are outstanding this tap's fragments are complete
            if constexpr (tap + 1 < NT) read_frags(std::integral_constant<int, (tap + 1 < NT ? tap + 1 : tap)>{}, b ^ 1);
            if constexpr (TP == 2) {
                if constexpr (tap + 1 < NT) asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(wf[b][0]), "+v"(wf[b][1]), "+v"(xf[b][0]), "+v"(xf[b][1]));
                else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wf[b][0]), "+v"(wf[b][1]), "+v"(xf[b][0]), "+v"(xf[b][1]));
            } else {
                if constexpr (tap + 1 < NT) asm volatile("s_waitcnt lgkmcnt(3)" : "+v"(wf[b][0]), "+v"(wf[b][1]), "+v"(xf[b][0]));
                else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wf[b][0]), "+v"(wf[b][1]), "+v"(xf[b][0]));
            }
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int j = 0; j < TP; j++)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[b][i], xf[b][j], acc[i][j], 0, 0, 0);
        };
        read_frags(std::integral_constant<int, 0>{}, 0);
        for_each_tap(step, std::make_integer_sequence<int, NT>{});
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // the next window has landed (this wave's part)
        __syncthreads();                                         // everybody's; and this window and its tables are free

        // ---- output: register v of a lane is channel cl + 32i + 16(v/8) + v%8 of its position, scaled
        //      and biased per channel
        const bool relu = a.act == ACT_RELU;
#pragma unroll
        for (int i = 0; i < TC; i++)
#pragma unroll
            for (int k = 0; k < 2; k++) {
                const int cb = 32 * i + 16 * k + 8 * lhalf;
                const f32x4 sq[2] = {*(const f32x4*)&scalel[cb], *(const f32x4*)&scalel[cb + 4]};
                const f32x4 bq[2] = {*(const f32x4*)&biasl[cb], *(const f32x4*)&biasl[cb + 4]};
#pragma unroll
                for (int j = 0; j < TP; j++) {
                    float v[8];
#pragma unroll
                    for (int e = 0; e < 8; e++) v[e] = fmaf(acc[i][j][8 * k + e], sq[e >> 2][e & 3], bq[e >> 2][e & 3]);
                    if (!relu) apply_act_n<8>(v, a.act);
                    uint32_t o[4];
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        o[q] = pack_bf16x2(v[2 * q], v[2 * q + 1]);
                        // relu on the rounded pair: a negative bf16 is a negative 16-bit integer
                        typedef short s16x2 __attribute__((ext_vector_type(2)));
                        const s16x2 z = {0, 0};
                        if (relu) o[q] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, o[q]), z));
                    }
                    const int co = cl + 32 * i + 16 * k;
                    const unsigned yo = pout[j] >= 0 && co < a.cout ? (unsigned)(pout[j] * a.y.stride + a.y.c0 + co) * 2u : OOBS;
                    __builtin_amdgcn_raw_buffer_store_b128(u32x4{o[0], o[1], o[2], o[3]}, yres, yo, 0, 0);
                }
            }
    }
}

// ---- host side -----------------------------------------------------------------------------
constexpr int TAPS_LDS_LIMIT = 160 * 1024;

struct TapsPlan { int bp, hrows, gh, gw, wgs; size_t bytes; };
constexpr int TAPS_CUS = 256;

// Whether (and how) this layer runs here: 16 stored input channels, stride 1, a 2x2 or 4x4
// filter, no residual.
static bool taps_plan(const ConvArgs& a, int nb, int G, TapsPlan* pl) {
    if (a.cin != 16 || a.sh != 1 || a.sw != 1 || a.pre_scale || a.res.p || a.cout % 8) return false;
    if (!((a.kh == 4 && a.kw == 4) || (a.kh == 2 && a.kw == 2))) return false;
    const int pb = a.Ho - 1 + a.kh - a.pt - a.H, pr = a.Wo - 1 + a.kw - a.pl - a.W;   // bottom / right padding
    if (a.Ho > a.H || a.Wo > a.W) return false;      // output positions are a subset of the input raster
    pl->gh = a.pt > pb ? a.pt : (pb > 0 ? pb : 0);
    pl->gw = a.pl > pr ? a.pl : (pr > 0 ? pr : 0);
    // 32-bit byte offsets into x and y, with 2^31 standing for 'outside'
    if ((long long)nb * a.H * a.W * a.x.stride * 2 >= 0x7FFFFF00LL) return false;
    if ((long long)nb * a.Ho * a.Wo * a.y.stride * 2 >= 0x7FFFFF00LL) return false;
    const long long PP = (long long)nb * (a.H + pl->gh) * (a.W + pl->gw);
    if (PP >= (1LL << 24)) return false;
    pl->bp = 256;
    const int need = pl->bp + (a.kh - 1) * (a.W + pl->gw) + a.kw;
    pl->hrows = (need + 127) / 128 * 128;
    pl->bytes = (size_t)a.kh * a.kw * 64 * 32 + 2 * ((size_t)pl->hrows * 32 + (size_t)pl->hrows * 4 + (size_t)pl->bp * 4) + 2 * 64 * 4;
    if (pl->bytes > (size_t)TAPS_LDS_LIMIT) return false;
    // As many workgroups as the chip holds at once, shared by the gang and the channel tiles, and
    // not one more: a workgroup that has to wait for a free slot starts its whole share of the
    // tiles when the others are finishing (measured: 171 instead of 170 per member costs 45 %).
    const int per_cu = (int)((size_t)TAPS_LDS_LIMIT / pl->bytes) < 1 ? 1 : (int)((size_t)TAPS_LDS_LIMIT / pl->bytes);
    const int ctiles = (a.cout + 63) / 64;
    long long wgs = ((long long)TAPS_CUS * per_cu) / ((long long)G * ctiles);
    if (wgs < 1) wgs = 1;
    const long long tiles = (PP + pl->bp - 1) / pl->bp;
    pl->wgs = (int)(wgs < tiles ? wgs : tiles);
    return true;
}

bool conv_taps_applicable(const ConvArgs& a, int nb) {
    TapsPlan pl;
    return taps_plan(a, nb, 1, &pl);
}

const char* conv_taps_name(const ConvArgs& a) { return a.kh == 4 ? "conv_taps16_bf16<256,4x4>" : "conv_taps16_bf16<256,2x2>"; }

template <int BP, int KH, int KW>
static hipError_t launch_taps_variant(const ConvArgs& a, const ConvArgs* argv, int G, int nb, const TapsPlan& pl, hipStream_t s) {
    static bool raised = false;                                  // LDS above 64 KB has to be asked for once
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void*)&conv_taps16_bf16<BP, KH, KW>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, TAPS_LDS_LIMIT);
        if (e != hipSuccess) return e;
        raised = true;
    }
    int wgs = pl.wgs;
    const dim3 grid((unsigned)wgs, (unsigned)((a.cout + 63) / 64), G);
    ENS_LAUNCH((conv_taps16_bf16<BP, KH, KW>), grid, dim3(256), pl.bytes, s, argv, nb, pl.hrows, pl.gh, pl.gw);
    return hipGetLastError();
}

hipError_t launch_conv_taps(const ConvArgs& a, const ConvArgs* argv, int G, int nb, hipStream_t s) {
    TapsPlan pl;
    if (!taps_plan(a, nb, G, &pl)) return hipErrorInvalidValue;
    if (a.x.stride % 8 || a.x.c0 % 8 || a.y.stride % 8 || a.y.c0 % 8) return hipErrorInvalidValue;
    if (a.kh == 4) return launch_taps_variant<256, 4, 4>(a, argv, G, nb, pl, s);
    return launch_taps_variant<256, 2, 2>(a, argv, G, nb, pl, s);
}

}  // namespace ens
