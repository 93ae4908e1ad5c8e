// A residual bottleneck as one kernel on the CDNA4 matrix cores: 1x1 convolution (cin -> C), 3x3
// stride-1 padding-1 convolution (C -> C) and 1x1 convolution (C -> cout, with the block's residual),
// each with its bias and activation, for C = 64 and C = 128.  The two C-channel tensors between
// the convolutions never leave the compute unit: run one after the other, the three layers write
// and read them through HBM, which at these widths is most of the block's traffic.
//
// Pixels are numbered in the padded raster of conv_halo.hip (one extra column per row, one extra
// row per image, treated as zeros), so that tap (dh, dw) of any position lies dh * (W + 1) + dw
// positions further on.  A workgroup of four wavefronts owns 128 consecutive positions and works
// in three phases:
//   1. t1 = act(W1 x + b1) for the R positions the 3x3 taps of the tile reach (the tile and W + 2
//      positions either side), 32 input channels at a time through a three-deep ring of input
//      chunks filled by asynchronous global-to-LDS loads; the result goes to LDS as bf16 in the
//      layout the 3x3 kernel reads its window in, with zeros at the positions that hold no pixel
//      (the 3x3 padding is zero in t1, not act(b1));
//   2. t2 = act(W2 * t1 + b2), nine taps over the window in LDS; the result replaces t1 in LDS;
//   3. y = act(W3 t2 + b3 + residual), 128 output channels at a time, stored from the accumulators.
// The weights do not pass through LDS: the member keeps a second copy of them in the order of the
// matrix-core operands (blocks of 32 rows x 16 columns, 16 bytes per lane), so a wavefront fetches
// a fragment as 1 KB in a row straight into registers, several steps ahead of its use.  Phases 2
// and 3 therefore run without a barrier; their only LDS traffic is the pixel fragments.
// The weight rows are handed to the matrix cores with bits 2 and 3 of the row number swapped, so
// that a lane of a 32x32 result block holds two runs of 8 consecutive channels of one position:
// 16-byte LDS writes in phases 1 and 2, 16-byte global stores in phase 3.  The price of the fusion
// is phase 1 on the R - 128 extra positions; the gain is the traffic of t1 and t2 and the second
// pass over x (the residual is re-read while its lines are still in a cache).
#include "conv_direct.h"


namespace ens {

constexpr int bn_max3(int a, int b, int c) { return a > b ? (a > c ? a : c) : (b > c ? b : c); }

constexpr int BN_BP = 128;           // positions per workgroup
constexpr int BN_NCH = 128;          // output channels per pass of phase 3
constexpr int BN_NXB = 3;            // input chunks in flight or in use
template <int C, int R>
constexpr int bn_big() { return bn_max3(BN_NXB * R * 64, (C / 64) * R * 128, (C / 64) * BN_BP * 128); }

// argv: the argument blocks of the three convolutions, gridDim.z of each (one per member of the gang)
template <int C, int R>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void bottleneck_bf16(const ConvArgs* __restrict__ argv, const int nb_) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int G = gridDim.z;
    const ConvArgs a1 = argv[blockIdx.z], a2 = argv[G + blockIdx.z], a3 = argv[2 * G + blockIdx.z];
    static_assert(C == 64 || C == 128, "64 or 128 channels between the convolutions");
    constexpr int BP = BN_BP, NCH = BN_NCH;
    // phase 1: wavefronts WR1 along the window rows, WC1 along the channels (a weight fragment is then
    // fetched by two wavefronts, not by all four)
    constexpr int WR1 = 2, WC1 = 4 / WR1;
    constexpr int TP1 = R / (32 * WR1), TC1 = C / (32 * WC1);
    static_assert(TP1 * 32 * WR1 == R && TC1 * 32 * WC1 == C && R % 64 == 0, "window rows split evenly");
    constexpr int XO = R / 64, WO = 2 * TC1;         // loads per thread and chunk: input rows, weight fragments
    // phases 2 and 3: 2 x 2 wavefronts, 64 positions each
    constexpr int TC2 = C / 64;
    constexpr int KK = C / 16;                       // matrix-core steps over C channels
    constexpr int PW = 8 / TC2;                      // steps the weight fragments are asked for ahead in phase 2
    constexpr int XS = R * 64;                       // bytes of an input chunk: R rows of 32 channels
    constexpr int T1B = R * 128, T2B = BP * 128;     // bytes of a 64-channel block of t1 / t2
    constexpr int BIG = bn_big<C, R>();

    const int W1 = a1.W + 1, H1 = a1.H + 1;
    const int PP = nb_ * H1 * W1;
    const int t = threadIdx.x, lane = t & 63, lrow = lane & 31, lhalf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int n_ptiles = (PP + BP - 1) / BP;
    int ptile, ctile;
    tile_of_block(n_ptiles, 1, &ptile, &ctile);
    const int pp0 = ptile * BP;
    const int cin1 = a1.cin, cout3 = a3.cout;

    // LDS: x chunks, then t1, then t2 | window row -> pixel index (-1: none) | biases of the three layers | their scales
    unsigned char* const big = lds;
    int* const tbl = (int*)(big + BIG);
    float* const b1l = (float*)(tbl + R);
    float* const b2l = b1l + C;
    float* const b3l = b2l + C;
    const int SBS = 2 * C + cout3;                               // from a channel's bias to its scale
    // the weights of the first two input chunks are asked for before anything else
    const int NS1 = (cin1 + 63) / 64 * 4, nk1 = cin1 / 32;       // steps per block of 32 weight rows (columns padded to 64s); input chunks
    const __amdgpu_buffer_rsrc_t w1res = __builtin_amdgcn_make_buffer_rsrc((void*)a1.wpk, 0, (int)((unsigned)C * (unsigned)(NS1 * 16) * 2u), 0x00020000);
    const int row0 = (wave % WR1) * (TP1 * 32), ch0 = (wave / WR1) * (TC1 * 32);   // phase 1: this wave's window rows and channels
    const unsigned wv1 = (unsigned)((ch0 / 32) * NS1 * 1024 + lane * 16);
    bf16x8 w0[2][TC1], w1[2][TC1], w2[2][TC1];                   // weights of this chunk, the next, the one after
    auto load_w = [&](bf16x8 (&w)[2][TC1], int kc) {
#pragma unroll
        for (int ks = 0; ks < 2; ks++)
#pragma unroll
            for (int i = 0; i < TC1; i++) w[ks][i] = bn_wload(w1res, wv1, (i * NS1 + kc * 2 + ks) * 1024);
    };
    load_w(w0, 0);
    if (nk1 > 1) load_w(w1, 1);
    // biases and scales are asked for at once and stored behind the first input chunks' loads (a loop of load
    // and store here would cost a round trip to memory per turn before the first input is asked for)
    static_assert(C <= 256, "one thread per middle channel");
    constexpr int NB3 = 2048 / 256;                              // the launcher admits up to 2048 output channels
    const bool mid_ok = t < C;
    const float b1_r = mid_ok ? ENS_GLOBAL(float, a1.bias)[t] : 0.f, s1_r = mid_ok ? ENS_GLOBAL(float, a1.scale)[t] : 0.f;
    const float b2_r = mid_ok ? ENS_GLOBAL(float, a2.bias)[t] : 0.f, s2_r = mid_ok ? ENS_GLOBAL(float, a2.scale)[t] : 0.f;
    float b3_r[NB3], s3_r[NB3];
#pragma unroll
    for (int j = 0; j < NB3; j++) {
        const int i = t + 256 * j;
        b3_r[j] = i < cout3 ? ENS_GLOBAL(float, a3.bias)[i] : 0.f;
        s3_r[j] = i < cout3 ? ENS_GLOBAL(float, a3.scale)[i] : 0.f;
    }
    raster_table(tbl, R, pp0 - (W1 + 1), PP, H1, W1, a1.H, a1.W);
    __syncthreads();

    // ---- load side.  Offsets past the end of a buffer give zeros in LDS (loads) or are dropped
    //      (stores); 2^31 is past the end of every buffer the launcher admits.
    constexpr unsigned OOBV = 0x80000000u;
    const unsigned npix = (unsigned)nb_ * (unsigned)(a1.H * a1.W);
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc((void*)a1.x.p, 0, (int)(npix * (unsigned)a1.x.stride * 2u), 0x00020000);
    const __amdgpu_buffer_rsrc_t w2res = __builtin_amdgcn_make_buffer_rsrc((void*)a2.wpk, 0, (int)(9u * C * C * 2u), 0x00020000);
    const __amdgpu_buffer_rsrc_t w3res = __builtin_amdgcn_make_buffer_rsrc((void*)a3.wpk, 0, (int)((unsigned)cout3 * (unsigned)C * 2u), 0x00020000);
    // thread roles in a load instruction of the workgroup (4 KB of 64-byte rows): row and swizzled chunk
    const int r4 = t >> 2, c4 = (t & 3) ^ ((r4 >> 2) & 3);
    unsigned xvo[XO];
#pragma unroll
    for (int s = 0; s < XO; s++) {
        const int p = tbl[r4 + 64 * s];
        xvo[s] = p >= 0 ? (unsigned)(p * a1.x.stride * 2) + (unsigned)(a1.x.c0 * 2 + c4 * 16) : OOBV;
    }
    unsigned char* const mine = lds + wave * 1024;               // this wave's quarter of a 4 KB load
    auto issue_x = [&](int buf, int kc) {
#pragma unroll
        for (int s = 0; s < XO; s++)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (lds_ptr_t)(mine + buf * XS + s * 4096), LDS_LOAD_BYTES, xvo[s], kc * 64, 0, 0);
    };

    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
    // phases 2 and 3: this wave's 64 positions and its half of the channels; the first weight fragments
    // of a phase are asked for before the phase before it has written its result to LDS
    const int wp0 = (wave & 1) * 64, wcg = wave >> 1;
    constexpr int NST = 9 * KK, PW3 = 4;
    static_assert(KK % PW3 == 0, "a step of phase 3 keeps its slot from pass to pass");
    const int wc2 = wcg * (32 * TC2), wc3 = wcg * 64;
    const unsigned wv2 = (unsigned)((wc2 / 32) * NST * 1024 + lane * 16);
    const unsigned wv3 = (unsigned)((wc3 / 32) * KK * 1024 + lane * 16);
    bf16x8 wq2[PW][TC2], wq3[PW3][2];
    // block i, step kk of pass nc of phase 3 lies at ((4 nc + wc3 / 32 + i) KK + kk) KB
    auto load_w3 = [&](bf16x8 (&w)[2], int nc, int kk) {
#pragma unroll
        for (int i = 0; i < 2; i++) w[i] = bn_wload(w3res, wv3, ((nc * (NCH / 32) + i) * KK + kk) * 1024);
    };

    // ---- phase 1: t1 over the window.  Chunk kc + 2 of the input and the weights of chunk kc + 2 are
    //      asked for while chunk kc is used.  Loads complete in the order they were issued, so the
    //      wait before a chunk is used counts what was issued after it and may still be on its way.
    {
        const int xr = row0 + lrow;
        const uint32_t xs1 = lds0 + (uint32_t)(xr * 64 + ((lhalf ^ ((xr >> 2) & 3)) << 4));
        f32x16 acc[TC1][TP1];
#pragma unroll
        for (int i = 0; i < TC1; i++)
#pragma unroll
            for (int j = 0; j < TP1; j++) bn_zero(acc[i][j]);
        issue_x(0, 0);
        if (nk1 > 1) issue_x(1, 1);
        // the tables' first readers come behind the barriers of the chunk loop
        if (mid_ok) {
            b1l[t] = b1_r;
            b2l[t] = b2_r;
            b1l[SBS + t] = s1_r;
            b2l[SBS + t] = s2_r;
        }
#pragma unroll
        for (int j = 0; j < NB3; j++) {
            const int i = t + 256 * j;
            if (i < cout3) {
                b3l[i] = b3_r[j];
                b3l[SBS + i] = s3_r[j];
            }
        }
        // One chunk: `wc` holds its weights, `wl` receives those of chunk kc + 2, BUF is its place in the
        // ring.  The three roles rotate with period three, so the loop below is written out three chunks
        // at a time: a rotation through register copies would have to wait for the loads just issued.
        auto chunk = [&](auto buf_c, bf16x8 (&wc)[2][TC1], bf16x8 (&wl)[2][TC1], const int kc) {
            constexpr int buf = decltype(buf_c)::value;
            // chunk kc has landed (this wave's part; with the barrier everybody's), and nobody still reads
            // the buffer that chunk kc + 2 goes to
            if (kc == 0) {
                if (nk1 > 1) bn_wait_vm<XO>(); else bn_wait_vm<0>();
            } else {
                if (kc + 1 < nk1) bn_wait_vm<WO + XO>(); else bn_wait_vm<0>();
            }
            __builtin_amdgcn_s_barrier();
            if (kc + 2 < nk1) {
                load_w(wl, kc + 2);
                issue_x((buf + 2) % 3, kc + 2);
            }
            const uint32_t xs = xs1 + (uint32_t)(buf * XS);
            bf16x8 xf[2][TP1];
            bn_unroll<TP1>([&](auto j) { xf[0][decltype(j)::value] = bn_lds_read<decltype(j)::value * 2048>(xs); });
            bn_unroll<TP1>([&](auto j) { xf[1][decltype(j)::value] = bn_lds_read<decltype(j)::value * 2048>(xs ^ 32u); });
            asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(TP1) : "memory");
#pragma unroll
            for (int j = 0; j < TP1; j++) bn_tie(xf[0][j]);
#pragma unroll
            for (int i = 0; i < TC1; i++)
#pragma unroll
                for (int j = 0; j < TP1; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wc[0][i], xf[0][j], acc[i][j], 0, 0, 0);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int j = 0; j < TP1; j++) bn_tie(xf[1][j]);
#pragma unroll
            for (int i = 0; i < TC1; i++)
#pragma unroll
                for (int j = 0; j < TP1; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wc[1][i], xf[1][j], acc[i][j], 0, 0, 0);
        };
        int kc = 0;
        for (; kc + 2 < nk1; kc += 3) {
            chunk(std::integral_constant<int, 0>{}, w0, w2, kc);
            chunk(std::integral_constant<int, 1>{}, w1, w0, kc + 1);
            chunk(std::integral_constant<int, 2>{}, w2, w1, kc + 2);
        }
        if (kc < nk1) chunk(std::integral_constant<int, 0>{}, w0, w2, kc);
        if (kc + 1 < nk1) chunk(std::integral_constant<int, 1>{}, w1, w0, kc + 1);
        bn_unroll<PW>([&](auto s) {
#pragma unroll
            for (int i = 0; i < TC2; i++) wq2[decltype(s)::value][i] = bn_wload(w2res, wv2, (i * NST + decltype(s)::value) * 1024);
        });
        __syncthreads();                                         // everybody is done with the input chunks
#pragma unroll
        for (int j = 0; j < TP1; j++) {
            const int row = row0 + 32 * j + lrow;
            const bool live = tbl[row] >= 0;
#pragma unroll
            for (int i = 0; i < TC1; i++)
#pragma unroll
                for (int k = 0; k < 2; k++) {
                    const int ch = ch0 + 32 * i + 16 * k + 8 * lhalf;
                    const u32x4 o = bn_pack(acc[i][j], k, a1.act, b1l + ch0 + 32 * i + 8 * lhalf, SBS);
                    *(u32x4*)(big + (ch >> 6) * T1B + row * 128 + ((((ch & 63) >> 3) ^ ((row >> 1) & 7)) << 4)) =
                        live ? o : u32x4{0u, 0u, 0u, 0u};
                }
        }
    }

    // What phase 3 needs from memory per pass, the residual of this lane's 2 x 2 x 2 runs of 8 channels,
    // is asked for a pass ahead; the first pass's now, before phase 2.
    const bool has_res = a3.res.p != nullptr;
    const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc((void*)a3.y.p, 0, (int)(npix * (unsigned)a3.y.stride * 2u), 0x00020000);
    const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(has_res ? a3.res.p : a3.y.p), 0, (int)(npix * (unsigned)(has_res ? a3.res.stride : a3.y.stride) * 2u), 0x00020000);
    unsigned yo[2], ro[2];
    {
        const int* own = tbl + W1 + 1 + wp0 + lrow;              // the centre tap's rows: this tile's outputs
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const int pout = own[32 * j];
            yo[j] = pout >= 0 ? (unsigned)(pout * a3.y.stride * 2) + (unsigned)((a3.y.c0 + wc3 + 8 * lhalf) * 2) : OOBV;
            ro[j] = pout >= 0 ? (unsigned)(pout * a3.res.stride * 2) + (unsigned)((a3.res.c0 + wc3 + 8 * lhalf) * 2) : OOBV;
        }
    }
    u32x4 resn[2][2][2];
    auto load_res = [&](int nc) {
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int k = 0; k < 2; k++)
                    resn[j][i][k] = __builtin_amdgcn_raw_buffer_load_b128(rres, ro[j], (nc * NCH + 32 * i + 16 * k) * 2, 0);
    };
    if (has_res) load_res(0);
    // ---- phase 2: t2 = 3x3 over t1.  No barrier and no LDS traffic but the pixel fragments: the
    //      weights come PW steps ahead from memory into registers.
    {
        f32x16 acc[TC2][2];
#pragma unroll
        for (int i = 0; i < TC2; i++)
#pragma unroll
            for (int j = 0; j < 2; j++) bn_zero(acc[i][j]);
        uint32_t xoff[9];                                        // tap (dh, dw): dh rows of the padded raster down, dw positions right
#pragma unroll
        for (int tap = 0; tap < 9; tap++) {
            const uint32_t q = (uint32_t)(wp0 + lrow + (tap / 3) * W1 + tap % 3);
            xoff[tap] = lds0 + q * 128 + ((((uint32_t)lhalf) ^ ((q >> 1) & 7)) << 4);
        }
        __syncthreads();                                         // t1 is complete
        bf16x8 xf[2][2];
        auto read_frags = [&](auto st_c, auto b_c) {
            constexpr int st = decltype(st_c)::value, b = decltype(b_c)::value;
            constexpr int tap = st / KK, kk = st % KK;           // step kk of the tap: block kk / 4 of t1, chunks 2 (kk % 4) and + 1
            const uint32_t xa = (xoff[tap] + (uint32_t)((kk / 4) * T1B)) ^ (uint32_t)((kk % 4) << 5);
            xf[b][0] = bn_lds_read<0>(xa);
            xf[b][1] = bn_lds_read<4096>(xa);
        };
        read_frags(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        bn_unroll<NST>([&](auto st_c) {
            constexpr int st = decltype(st_c)::value, b = st & 1, slot = st % PW;
            if constexpr (st + 1 < NST) {
                read_frags(std::integral_constant<int, st + 1>{}, std::integral_constant<int, b ^ 1>{});
                asm volatile("s_waitcnt lgkmcnt(2)" ::: "memory");
            } else {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
            bn_tie(xf[b][0]);
            bn_tie(xf[b][1]);
            bf16x8 wc[TC2];
#pragma unroll
            for (int i = 0; i < TC2; i++) wc[i] = wq2[slot][i];
            if constexpr (st + PW < NST) {
#pragma unroll
                for (int i = 0; i < TC2; i++) wq2[slot][i] = bn_wload(w2res, wv2, (i * NST + st + PW) * 1024);
            }
#pragma unroll
            for (int i = 0; i < TC2; i++)
#pragma unroll
                for (int j = 0; j < 2; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wc[i], xf[b][j], acc[i][j], 0, 0, 0);
        });
#pragma unroll
        for (int kk = 0; kk < PW3; kk++) load_w3(wq3[kk], 0, kk);
        __syncthreads();                                         // everybody is done with t1
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const int row = wp0 + 32 * j + lrow;
#pragma unroll
            for (int i = 0; i < TC2; i++)
#pragma unroll
                for (int k = 0; k < 2; k++) {
                    const int ch = wc2 + 32 * i + 16 * k + 8 * lhalf;
                    *(u32x4*)(big + (ch >> 6) * T2B + row * 128 + ((((ch & 63) >> 3) ^ ((row >> 1) & 7)) << 4)) =
                        bn_pack(acc[i][j], k, a2.act, b2l + wc2 + 32 * i + 8 * lhalf, SBS);
                }
        }
    }

    // ---- phase 3: y = W3 t2 + residual, 128 channels per pass.  Register v of a lane is channel
    //      16(v/8) + 8(lane/32) + v%8 of its block and position; stores to positions without a pixel
    //      carry the out-of-range offset and are dropped by the hardware.
    {
        const int xr = wp0 + lrow;
        const uint32_t xs3 = lds0 + (uint32_t)(xr * 128 + ((lhalf ^ ((xr >> 1) & 7)) << 4));
        const int nch = cout3 / NCH;
        const bool relu = a3.act == ACT_RELU;
        // weight fragments PW3 steps ahead, on into the next pass
        __syncthreads();                                         // t2 is complete
        for (int nc = 0; nc < nch; nc++) {
            u32x4 res[2][2][2];
#pragma unroll
            for (int j = 0; j < 2; j++)
#pragma unroll
                for (int i = 0; i < 2; i++)
#pragma unroll
                    for (int k = 0; k < 2; k++) res[j][i][k] = resn[j][i][k];
            if (has_res && nc + 1 < nch) load_res(nc + 1);
            f32x16 acc[2][2];
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int j = 0; j < 2; j++) bn_zero(acc[i][j]);
            bf16x8 xf[2][2];
            auto read_frags = [&](auto kk_c, auto b_c) {
                constexpr int kk = decltype(kk_c)::value, b = decltype(b_c)::value;
                const uint32_t xa = (xs3 + (uint32_t)((kk / 4) * T2B)) ^ (uint32_t)((kk % 4) << 5);
                xf[b][0] = bn_lds_read<0>(xa);
                xf[b][1] = bn_lds_read<4096>(xa);
            };
            read_frags(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
            bn_unroll<KK>([&](auto kk_c) {
                constexpr int kk = decltype(kk_c)::value, b = kk & 1;
                if constexpr (kk + 1 < KK) {
                    read_frags(std::integral_constant<int, kk + 1>{}, std::integral_constant<int, b ^ 1>{});
                    asm volatile("s_waitcnt lgkmcnt(2)" ::: "memory");
                } else {
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                }
                bn_tie(xf[b][0]);
                bn_tie(xf[b][1]);
                constexpr int slot = kk % PW3;
                bf16x8 wc[2] = {wq3[slot][0], wq3[slot][1]};
                if constexpr (kk + PW3 < KK) {
                    load_w3(wq3[slot], nc, kk + PW3);
                } else {
                    if (nc + 1 < nch) load_w3(wq3[slot], nc + 1, kk + PW3 - KK);
                }
#pragma unroll
                for (int i = 0; i < 2; i++)
#pragma unroll
                    for (int j = 0; j < 2; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wc[i], xf[b][j], acc[i][j], 0, 0, 0);
            });
#pragma unroll
            for (int j = 0; j < 2; j++)
#pragma unroll
                for (int i = 0; i < 2; i++)
#pragma unroll
                    for (int k = 0; k < 2; k++) {
                        float v[8];
                        bn_affine8(v, acc[i][j], k, b3l + nc * NCH + wc3 + 32 * i + 8 * lhalf, SBS);
                        if (has_res) {
                            const uint32_t rr[4] = {res[j][i][k].x, res[j][i][k].y, res[j][i][k].z, res[j][i][k].w};
#pragma unroll
                            for (int q = 0; q < 4; q++) {
                                v[2 * q] += bf16_to_f32((uint16_t)(rr[q] & 0xFFFF));
                                v[2 * q + 1] += bf16_to_f32((uint16_t)(rr[q] >> 16));
                            }
                        }
                        if (!relu) apply_act_n<8>(v, a3.act);
                        uint32_t o[4];
#pragma unroll
                        for (int q = 0; q < 4; q++) {
                            o[q] = pack_bf16x2(v[2 * q], v[2 * q + 1]);
                            if (relu) {                          // on the rounded pair: a negative bf16 is a negative 16-bit integer
                                typedef short s16x2 __attribute__((ext_vector_type(2)));
                                const s16x2 z = {0, 0};
                                o[q] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, o[q]), z));
                            }
                        }
                        __builtin_amdgcn_raw_buffer_store_b128(u32x4{o[0], o[1], o[2], o[3]}, yres, yo[j], (nc * NCH + 32 * i + 16 * k) * 2, 0);
                    }
        }
    }
}

// ---- host side -----------------------------------------------------------------------------
constexpr int BNECK_LDS_LIMIT = 160 * 1024;
constexpr int BNECK_MIN_TILES = 24;

struct BneckPlan { int c, rows; size_t bytes; int tiles; };

static bool bneck_plan(const ConvArgs& a1, const ConvArgs& a2, const ConvArgs& a3, int nb, BneckPlan* pl) {
    auto pointwise = [](const ConvArgs& a) {
        return a.kh == 1 && a.kw == 1 && a.sh == 1 && a.sw == 1 && a.pt == 0 && a.pl == 0 && a.Ho == a.H && a.Wo == a.W && !a.pre_scale;
    };
    if (!pointwise(a1) || !pointwise(a3) || a1.res.p || a2.res.p) return false;
    if (a2.kh != 3 || a2.kw != 3 || a2.sh != 1 || a2.sw != 1 || a2.pt != 1 || a2.pl != 1 || a2.pre_scale) return false;
    if (a2.H != a1.H || a2.W != a1.W || a2.Ho != a1.H || a2.Wo != a1.W || a3.H != a1.H || a3.W != a1.W) return false;
    const int c = a1.cout;
    if ((c != 64 && c != 128) || a2.cin != c || a2.cout != c || a3.cin != c) return false;
    if (a1.cin % 32 || a3.cout % BN_NCH || a3.cout > 2048 || !a1.wpk || !a2.wpk || !a3.wpk) return false;
    // the middle tensors are skipped: the 3x3 reads what the first convolution writes, and so on
    if (a2.x.p != a1.y.p || a2.x.c0 != a1.y.c0 || a3.x.p != a2.y.p || a3.x.c0 != a2.y.c0) return false;
    if (a3.y.p == a1.x.p) return false;
    // 32-bit byte offsets with 2^31 standing for 'outside'; float index arithmetic is exact below 2^24
    const long long P = (long long)nb * a1.H * a1.W;
    if (P * a1.x.stride * 2 >= 0x7FFFFF00LL || P * a3.y.stride * 2 >= 0x7FFFFF00LL) return false;
    if (a3.res.p && P * a3.res.stride * 2 >= 0x7FFFFF00LL) return false;
    const long long PP = (long long)nb * (a1.H + 1) * (a1.W + 1);
    if (PP >= (1LL << 24)) return false;
    if (a1.x.stride % 8 || a1.x.c0 % 8 || a3.y.stride % 8 || a3.y.c0 % 8) return false;
    if (a3.res.p && (a3.res.stride % 8 || a3.res.c0 % 8)) return false;
    pl->c = c;
    pl->rows = c == 64 ? 256 : 192;
    if (BN_BP + 2 * (a1.W + 1) + 2 > pl->rows) return false;
    const int big = c == 64 ? bn_big<64, 256>() : bn_big<128, 192>();
    pl->bytes = (size_t)big + (size_t)pl->rows * 4 + (size_t)(2 * c + a3.cout) * 8;
    pl->tiles = (int)((PP + BN_BP - 1) / BN_BP);
    return pl->bytes <= (size_t)BNECK_LDS_LIMIT;
}

bool conv_bneck_applicable(const ConvArgs& a1, const ConvArgs& a2, const ConvArgs& a3, int nb, int G) {
    BneckPlan pl;
    if (!bneck_plan(a1, a2, a3, nb, &pl)) return false;
    // A workgroup runs its tile's three layers one after the other, so a handful of tiles leaves the
    // chip to a handful of workgroups; the separate kernels split the channels too.  Measured on a
    // ResNet-50-shaped member the one kernel wins from about two dozen tiles on (batch 4 at 28x28).
    long long least = BNECK_MIN_TILES;
    return (long long)pl.tiles * G >= least;
}

const char* conv_bneck_name(const ConvArgs& a1) { return a1.cout == 64 ? "bottleneck_bf16<c64>" : "bottleneck_bf16<c128>"; }

template <int C, int R>
static hipError_t launch_bneck_variant(const ConvArgs* argv, int G, int nb, const BneckPlan& pl, hipStream_t s) {
    static bool raised = false;                                  // LDS above 64 KB has to be asked for once
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void*)&bottleneck_bf16<C, R>, hipFuncAttributeMaxDynamicSharedMemorySize, BNECK_LDS_LIMIT);
        if (e != hipSuccess) return e;
        raised = true;
    }
    ENS_LAUNCH((bottleneck_bf16<C, R>), dim3((unsigned)pl.tiles, 1, G), dim3(256), pl.bytes, s, argv, nb);
    return hipGetLastError();
}

hipError_t launch_conv_bneck(const ConvArgs& a1, const ConvArgs& a2, const ConvArgs& a3, const ConvArgs* argv, int G, int nb, hipStream_t s) {
    BneckPlan pl;
    if (!bneck_plan(a1, a2, a3, nb, &pl)) return hipErrorInvalidValue;
    return pl.c == 64 ? launch_bneck_variant<64, 256>(argv, G, nb, pl, s) : launch_bneck_variant<128, 192>(argv, G, nb, pl, s);
}

}  // namespace ens
