// 3x3, stride 1, padding 1 convolution on the CDNA4 matrix cores with the filter held in
// registers, for layers with 64 input channels: a wavefront owns 32 output channels, whose
// 9 x 64 weights per channel are the A operands of 36 v_mfma_f32_32x32x16_bf16 steps, 144
// registers per lane, loaded once.  The workgroups are persistent: each walks over position
// tiles of its (member, channel tile), and all a tile needs from memory is its input window,
// which arrives in LDS by asynchronous loads while the previous tile is computed.  The inner loop
// is LDS reads of pixel fragments and matrix-core instructions only: no weight traffic, no
// barrier, no address arithmetic beyond one add per tap.
//
// Pixels are numbered in the padded raster of conv_halo.hip (one extra column per row, one extra
// row per image, loaded as zeros): tap (dh, dw) of any position lies dh * (W + 1) + dw positions
// further on.  The window of a tile takes 128 bytes of LDS per position, chunks swizzled as in
// the generic kernel.
//
// Wavefront roles in a workgroup of four: WPX along the positions, WCG along groups of 32 output
// channels.  Two workgroups share a compute unit (256 registers per lane each): while one sends
// its output off the other keeps the matrix cores busy.
//
// The output leaves straight from the accumulators.  A lane of a 32x32 result block holds one
// position and the matrix rows 8g + 4h + e (g = 0..3, e = 0..3, h = lane / 32); the weight rows
// are handed to the matrix cores with bits 2 and 3 of the row number swapped, so that those rows
// are the channels 16(g/2) + 8h + 4(g%2) + e: two runs of 8 consecutive channels, two 16-byte
// stores per lane, 32 contiguous bytes per position and instruction, after the per-channel scale
// and bias (both wait in LDS).  A tile therefore costs one barrier: the one that says that the next
// window has landed and the current one is free.
#include "conv_common.h"

#include <type_traits>
#include <utility>

namespace ens {

typedef __attribute__((address_space(3))) void* lds_ptr_t;

template <int OFFSET>
__device__ __forceinline__ bf16x8 wreg_lds_read(uint32_t addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
    return v;
}

template <class F, int... T>
__device__ __forceinline__ void wreg_for_each(F&& f, std::integer_sequence<int, T...>) {
    (f(std::integral_constant<int, T>{}), ...);
}

template <int BP, int WPX, int WCG>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void conv3x3_wreg_bf16(const ConvArgs* __restrict__ argv, const int nb_, const int hrows) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const ConvArgs a = argv[blockIdx.z];
    static_assert(WPX * WCG == 4, "four wavefronts per workgroup");
    constexpr int BC = 32 * WCG;                     // output channels of the workgroup
    constexpr int WTP = BP / WPX, TP = WTP / 32;     // positions per wave
    static_assert(TP >= 1 && TP <= 2, "32 or 64 positions per wave");
    constexpr int ROWB = 128, BLK = 32 * ROWB;
    constexpr int NSTEP = 9 * 4;                     // matrix-core steps per tile: 9 taps x 64 channels / 16

    const int W1 = a.W + 1, H1 = a.H + 1;
    const int PP = nb_ * H1 * W1;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int px_w = wave % WPX, cg_w = wave / WPX;
    const int wp0 = px_w * WTP, wc0 = cg_w * 32;
    const int n_ptiles = (PP + BP - 1) / BP;
    const int c0 = blockIdx.y * BC;
    const int hbytes = hrows * ROWB, nsl = hrows / 32;

    const TileWalk walk = tile_walk(n_ptiles, (blockIdx.y + blockIdx.z * gridDim.y) * gridDim.x);
    int ptile = walk.first;
    if (ptile >= walk.end) return;

    // LDS: window 0 | window 1 | three tables window row -> byte offset of the pixel in x (out of range: no
    // pixel) | three tables window row -> pixel index (-1: none) | bias, then scale, of the BC channels.  On its way
    // to the registers the filter passes through the FSTAGE bytes after window 0, which the tables keep
    // clear of.
    constexpr int FSTAGE = 5 * BC * 128;
    unsigned* const tblx = (unsigned*)(lds + (2 * hbytes > hbytes + FSTAGE ? 2 * hbytes : hbytes + FSTAGE));
    int* const tblp = (int*)(tblx + 3 * hrows);
    float* const biasl = (float*)(tblp + 3 * hrows);
    float* const scalel = biasl + BC;

    // ---- window loads.  Offsets past the end of a buffer give zeros in LDS (loads) or are dropped
    //      (stores); 2^31 is past the end of every buffer the launcher admits.
    constexpr unsigned OOBV = 0x80000000u;
    const unsigned nbytes_x = (unsigned)nb_ * (unsigned)(a.H * a.W) * (unsigned)a.x.stride * 2u;
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc((void*)a.x.p, 0, (int)nbytes_x, 0x00020000);
    const int r0 = t >> 3;
    const unsigned xlane = (unsigned)(a.x.c0 * 2 + (((t & 7) ^ ((r0 >> 1) & 7)) * 16));

    // Table row t of a tile is window position first + t, first = tile * BP - (W1 + 1).  Thread t
    // keeps that position as (image, row, column) and steps it from one of its tiles to the next
    // by a constant, so a table costs a few adds instead of two divisions per entry.
    const int img = H1 * W1;
    int tn, thi, twi;
    {
        const int pp = ptile * BP - (W1 + 1) + t + img;          // one image further on: never negative
        const float inv_img = __builtin_amdgcn_rcpf((float)img), inv_w1 = __builtin_amdgcn_rcpf((float)W1);
        int n = (int)((float)pp * inv_img);
        int rem = pp - n * img;
        n += (rem >= img ? 1 : 0) - (rem < 0 ? 1 : 0);
        rem = pp - n * img;
        int hi = (int)((float)rem * inv_w1);
        int wi = rem - hi * W1;
        hi += (wi >= W1 ? 1 : 0) - (wi < 0 ? 1 : 0);
        wi = rem - hi * W1;
        tn = n - 1; thi = hi; twi = wi;
    }
    const int step_tiles = walk.step;
    const int adv = step_tiles * BP;
    const int adv_n = adv / img, adv_h = (adv - adv_n * img) / W1, adv_w = adv - adv_n * img - adv_h * W1;
    // writes slot `slot` for the tile the thread's position stands at, then moves on to the next tile
    auto make_table = [&](int slot) {
        if (t < hrows) {
            const bool ok = (unsigned)tn < (unsigned)nb_ && thi < a.H && twi < a.W;
            const int pix = (tn * a.H + thi) * a.W + twi;
            tblx[slot * hrows + t] = ok ? (unsigned)(pix * a.x.stride * 2) : OOBV;
            tblp[slot * hrows + t] = ok ? pix : -1;
        }
        twi += adv_w;
        const int cw = twi >= W1 ? 1 : 0;
        twi -= cw ? W1 : 0;
        thi += adv_h + cw;
        const int ch = thi >= H1 ? 1 : 0;
        thi -= ch ? H1 : 0;
        tn += adv_n + ch;
    };
    auto issue_window = [&](int buf, int slot) {
        const unsigned* tbl = tblx + slot * hrows;
        unsigned char* dst = lds + buf * hbytes + wave * 1024;
        for (int s0 = 0; s0 < nsl; s0 += 8) {                    // eight table look-ups in flight at a time
            unsigned o8[8];
#pragma unroll
            for (int j = 0; j < 8; j++) o8[j] = tbl[min(s0 + j, nsl - 1) * 32 + r0];
#pragma unroll
            for (int j = 0; j < 8; j++) {
                if (s0 + j >= nsl) break;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (lds_ptr_t)(dst + (s0 + j) * 4096), LDS_LOAD_BYTES,
                                                         o8[j] + xlane, 0, 0, 0);
            }
        }
    };
    make_table(0);
    make_table(1);                                               // (of a tile past the end when there is only one: never used)
    if (t < BC) {
        biasl[t] = c0 + t < a.cout ? a.bias[c0 + t] : 0.f;
        scalel[t] = c0 + t < a.cout ? a.scale[c0 + t] : 1.f;
    }
    __syncthreads();
    issue_window(0, 0);

    // ---- the filter: fragment (tap, ks) of this wave's 32 channels.  A lane's 16 bytes lie in a
    //      different weight row than its neighbour's, so the rows come through LDS with coalesced
    //      asynchronous loads (taps 0..4 next to the first window, which arrives meanwhile, then
    //      taps 5..8) and are picked up from there.
    bf16x8 wreg[9][4];
    {
        const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
            (void*)a.w, 0, (int)((unsigned)a.cout * (unsigned)(9 * a.cin) * 2u), 0x00020000);
        unsigned wvo[BC / 32];                                   // weight row c0 + 32*i + r0, this thread's chunk
#pragma unroll
        for (int i = 0; i < BC / 32; i++) {
            const int ch = c0 + 32 * i + r0;
            wvo[i] = ch < a.cout ? (unsigned)ch * (unsigned)(9 * a.cin) * 2u + (unsigned)(((t & 7) ^ ((r0 >> 1) & 7)) * 16)
                                 : OOBV;
        }
        const int mrow = lane & 31;                              // matrix row; its channel has bits 2 and 3 swapped
        const int rho = wc0 + ((mrow & 0x13) | ((mrow & 4) << 1) | ((mrow & 8) >> 1));
        const uint32_t key = (uint32_t)((rho >> 1) & 7), lh = (uint32_t)(lane >> 5);
        unsigned char* const fst = lds + hbytes;
#pragma unroll
        for (int tap0 = 0; tap0 < 9; tap0 += 5) {
#pragma unroll
            for (int j = 0; j < 5; j++) {
                if (tap0 + j >= 9) break;
#pragma unroll
                for (int i = 0; i < BC / 32; i++)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(wres, (lds_ptr_t)(fst + j * BC * 128 + i * 4096 + wave * 1024),
                                                             LDS_LOAD_BYTES, wvo[i], (tap0 + j) * a.cin * 2, 0, 0);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 5; j++) {
                if (tap0 + j >= 9) break;
#pragma unroll
                for (int ks = 0; ks < 4; ks++)
                    wreg[tap0 + j][ks] = *(const bf16x8*)(fst + j * BC * 128 + rho * 128 + (((2 * ks + lh) ^ key) << 4));
            }
            __syncthreads();                                     // picked up: the stage is free for the next taps, then for window 1
        }
    }

    // ---- fragment side: lane reads position wp0 + (lane & 31) (+32) of the tap, chunk 2*ks + lane/32.
    //      The byte offsets of the nine taps inside a window do not depend on the tile.
    const int lrow = lane & 31, lhalf = lane >> 5;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
    uint32_t xoff[9];
#pragma unroll
    for (int tap = 0; tap < 9; tap++) {
        const uint32_t q = (uint32_t)(wp0 + lrow + (tap / 3) * W1 + tap % 3);
        xoff[tap] = q * ROWB + ((((uint32_t)lhalf) ^ ((q >> 1) & 7)) << 4);
    }
    // this lane's output channels: c0 + wc0 + 16k + 8*lhalf + 0..7 for k = 0, 1 (the launcher admits
    // multiples of 32 output channels only, so a wave's 32 channels exist or do not as a whole)
    const int cl = wc0 + 8 * lhalf;
    const bool wave_ok = c0 + wc0 < a.cout;
    const unsigned npix = (unsigned)nb_ * (unsigned)(a.H * a.W);
    const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.y.p, 0, (int)(npix * (unsigned)a.y.stride * 2u), 0x00020000);
    const bool has_res = a.res.p != nullptr;
    const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(has_res ? a.res.p : a.y.p), 0, (int)(npix * (unsigned)(has_res ? a.res.stride : a.y.stride) * 2u), 0x00020000);
    const unsigned ylane = (unsigned)((a.y.c0 + c0 + cl) * 2), rlane = (unsigned)((a.res.c0 + c0 + cl) * 2);

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");             // the first window has landed: this wave's part,
    __builtin_amdgcn_s_barrier();                                // and with the barrier everybody's

    // Per tile: ask for the next window, write the table of the tile after that, fetch this tile's
    // residual, compute, wait for the next window, send the output off.  The one wait counter
    // covers loads and stores alike, so the wait sits before this tile's stores are issued.
    int slot = 0;
    for (int buf = 0; ptile < walk.end; ptile += step_tiles, buf ^= 1) {
        const int slot1 = slot == 2 ? 0 : slot + 1, slot2 = slot1 == 2 ? 0 : slot1 + 1;
        if (ptile + step_tiles < walk.end) issue_window(buf ^ 1, slot1);
        // slot2 held the previous tile's table, which every wave has read before that tile's barrier
        make_table(slot2);
        const int* own = tblp + slot * hrows + W1 + 1 + wp0 + lrow;   // the centre tap's rows: this tile's outputs
        unsigned yo[TP], ro[TP];
#pragma unroll
        for (int j = 0; j < TP; j++) {
            const int pout = own[j * 32];
            yo[j] = pout >= 0 && wave_ok ? (unsigned)(pout * a.y.stride * 2) + ylane : OOBV;
            ro[j] = pout >= 0 && wave_ok ? (unsigned)(pout * a.res.stride * 2) + rlane : OOBV;
        }
        u32x4 res[TP][2];
        if (has_res) {
#pragma unroll
            for (int j = 0; j < TP; j++) {
                res[j][0] = __builtin_amdgcn_raw_buffer_load_b128(rres, ro[j], 0, 0);
                res[j][1] = __builtin_amdgcn_raw_buffer_load_b128(rres, ro[j], 32, 0);
            }
        }

        f32x16 acc[TP];
#pragma unroll
        for (int j = 0; j < TP; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[j][v] = 0.f;
        const uint32_t wbase = lds0 + (uint32_t)(buf * hbytes);
        bf16x8 xf[2][TP];
        auto read_frags = [&](auto step_c, int b) {
            constexpr int step = decltype(step_c)::value;
            constexpr int tap = step / 4, ks = step % 4;
            const uint32_t xa = (wbase + xoff[tap]) ^ (uint32_t)(ks << 5);
            xf[b][0] = wreg_lds_read<0>(xa);
            if (TP > 1) xf[b][1 % TP] = wreg_lds_read<BLK>(xa);
        };
        auto do_step = [&](auto step_c) {
            constexpr int step = decltype(step_c)::value;
            constexpr int tap = step / 4, ks = step % 4, b = step & 1;
            // the next step's reads are issued first; LDS returns in order, so once no more than
            // those are outstanding this step's fragments are complete
            if constexpr (step + 1 < NSTEP) read_frags(std::integral_constant<int, (step + 1 < NSTEP ? step + 1 : step)>{}, b ^ 1);
            if constexpr (TP == 2) {
                if constexpr (step + 1 < NSTEP) asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(xf[b][0]), "+v"(xf[b][1]));
                else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(xf[b][0]), "+v"(xf[b][1]));
            } else {
                if constexpr (step + 1 < NSTEP) asm volatile("s_waitcnt lgkmcnt(1)" : "+v"(xf[b][0]));
                else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(xf[b][0]));
            }
#pragma unroll
            for (int j = 0; j < TP; j++)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[tap][ks], xf[b][j], acc[j], 0, 0, 0);
        };
        read_frags(std::integral_constant<int, 0>{}, 0);
        wreg_for_each(do_step, std::make_integer_sequence<int, NSTEP>{});
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // the next window has landed (this wave's part)
        __syncthreads();                                         // everybody's; and this window is free for the one after

        // ---- output: register v of a lane is channel cl + 16(v/8) + v%8 of its position, scaled and
        //      biased per channel.  Stores to positions without a pixel carry the out-of-range offset
        //      and are dropped by the hardware.
        auto emit = [&](auto res_c, auto relu_c) {
            constexpr bool RES = decltype(res_c)::value, RELU = decltype(relu_c)::value;
#pragma unroll
            for (int k = 0; k < 2; k++) {
                const f32x4 sq[2] = {*(const f32x4*)&scalel[cl + 16 * k], *(const f32x4*)&scalel[cl + 16 * k + 4]};
                const f32x4 bq[2] = {*(const f32x4*)&biasl[cl + 16 * k], *(const f32x4*)&biasl[cl + 16 * k + 4]};
#pragma unroll
                for (int j = 0; j < TP; j++) {
                    float v[8];
#pragma unroll
                    for (int e = 0; e < 8; e++) v[e] = fmaf(acc[j][8 * k + e], sq[e >> 2][e & 3], bq[e >> 2][e & 3]);
                    if constexpr (RES) {
                        const uint32_t rr[4] = {res[j][k].x, res[j][k].y, res[j][k].z, res[j][k].w};
#pragma unroll
                        for (int q = 0; q < 4; q++) {
                            v[2 * q] += bf16_to_f32((uint16_t)(rr[q] & 0xFFFF));
                            v[2 * q + 1] += bf16_to_f32((uint16_t)(rr[q] >> 16));
                        }
                    }
                    if constexpr (!RELU) apply_act_n<8>(v, a.act);
                    uint32_t o[4];
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        o[q] = pack_bf16x2(v[2 * q], v[2 * q + 1]);
                        if constexpr (RELU) {
                            // relu on the rounded pair: a negative bf16 is a negative 16-bit integer
                            typedef short s16x2 __attribute__((ext_vector_type(2)));
                            const s16x2 z = {0, 0};
                            o[q] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, o[q]), z));
                        }
                    }
                    __builtin_amdgcn_raw_buffer_store_b128(u32x4{o[0], o[1], o[2], o[3]}, yres, yo[j], 32 * k, 0);
                }
            }
        };
        if (a.act == ACT_RELU) {
            if (has_res) emit(std::true_type{}, std::true_type{});
            else emit(std::false_type{}, std::true_type{});
        } else {
            if (has_res) emit(std::true_type{}, std::false_type{});
            else emit(std::false_type{}, std::false_type{});
        }
        slot = slot1;
    }
}

// ---- host side -----------------------------------------------------------------------------
constexpr int WREG_LDS_LIMIT = 160 * 1024;
constexpr int WREG_CUS = 256;

struct WregPlan { int hrows, wgs; size_t bytes; };

static bool wreg_plan(const ConvArgs& a, int nb, int G, WregPlan* pl) {
    if (a.kh != 3 || a.kw != 3 || a.sh != 1 || a.sw != 1 || a.pt != 1 || a.pl != 1) return false;
    if (a.Ho != a.H || a.Wo != a.W || a.pre_scale || a.cin != 64 || a.cout % 32) return false;
    // 32-bit byte offsets into x, y and the residual, with 2^31 standing for 'outside'
    if ((long long)nb * a.H * a.W * a.x.stride * 2 >= 0x7FFFFF00LL) return false;
    if ((long long)nb * a.H * a.W * a.y.stride * 2 >= 0x7FFFFF00LL) return false;
    if (a.res.p && (long long)nb * a.H * a.W * a.res.stride * 2 >= 0x7FFFFF00LL) return false;
    const long long PP = (long long)nb * (a.H + 1) * (a.W + 1);
    if (PP >= (1LL << 24)) return false;
    const int bp = 128;
    const int need = bp + 2 * (a.W + 1) + 2;
    pl->hrows = (need + 31) / 32 * 32;
    if (pl->hrows > 256) return false;                           // one table row per thread
    // two windows, or one window and the stage the filter passes through, whichever is larger; tables; bias and scale
    const size_t hb = (size_t)pl->hrows * 128, fstage = (size_t)5 * 64 * 128;
    pl->bytes = (2 * hb > hb + fstage ? 2 * hb : hb + fstage) + 6 * (size_t)pl->hrows * 4 + 2 * 64 * 4;
    if (2 * pl->bytes > (size_t)WREG_LDS_LIMIT) return false;
    // as many workgroups as the chip holds at once (two per compute unit), and not one more
    const int ctiles = (a.cout + 63) / 64;
    long long wgs = (2LL * WREG_CUS) / ((long long)G * ctiles);
    if (wgs < 1) wgs = 1;
    const long long tiles = (PP + bp - 1) / bp;
    pl->wgs = (int)(wgs < tiles ? wgs : tiles);
    return true;
}

bool conv_wreg_applicable(const ConvArgs& a, int nb, int G) {
    WregPlan pl;
    return wreg_plan(a, nb, G, &pl);
}

const char* conv_wreg_name(const ConvArgs&) { return "conv3x3_wreg_bf16<128,c64>"; }

hipError_t launch_conv_wreg(const ConvArgs& a, const ConvArgs* argv, int G, int nb, hipStream_t s) {
    WregPlan pl;
    if (!wreg_plan(a, nb, G, &pl)) return hipErrorInvalidValue;
    if (a.x.stride % 8 || a.x.c0 % 8 || a.y.stride % 8 || a.y.c0 % 8) return hipErrorInvalidValue;
    if (a.res.p && (a.res.stride % 8 || a.res.c0 % 8)) return hipErrorInvalidValue;
    static bool raised = false;                                  // LDS above 64 KB has to be asked for once
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void*)&conv3x3_wreg_bf16<128, 2, 2>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, WREG_LDS_LIMIT);
        if (e != hipSuccess) return e;
        raised = true;
    }
    int wgs = pl.wgs;
    const dim3 grid((unsigned)wgs, (unsigned)((a.cout + 63) / 64), G);
    ENS_LAUNCH((conv3x3_wreg_bf16<128, 2, 2>), grid, dim3(256), pl.bytes, s, argv, nb, pl.hrows);
    return hipGetLastError();
}

}  // namespace ens
