// A layer of a dense block as one kernel on the CDNA4 matrix cores: pre-activated 1x1 convolution
// (relu(x * scale + shift) per input channel, cin -> 128, bias, activation) followed by a 3x3
// stride-1 padding-1 convolution (128 -> 32) that appends its output to the block's tensor.  The
// 128-channel tensor in between stays in LDS.  Run one after the other the two layers are short
// launches (a dozen microseconds each at 14x14 and 7x7, whatever the batch): the kernel is there to
// halve their number, not to save traffic.
//
// Organisation as in conv_bneck.hip without its third phase.  Pixels are numbered in the padded
// raster (one extra column per row, one extra row per image, treated as zeros); a workgroup of
// four wavefronts owns 128 consecutive positions.  Phase 1 computes the first layer on the R
// positions the 3x3 taps of the tile reach, input in chunks of 32 channels through a three-deep
// ring of asynchronous global-to-LDS loads with counted waits; the pre-activation is applied in
// place to each chunk once it has landed (its scale and shift wait in LDS); the
// result goes to LDS as bf16 in the window layout of the 3x3 kernels, zeros where the raster holds
// no pixel.  Phase 2 is the nine taps, each wavefront 32 positions x 32 channels, stored from the
// accumulators.  On small maps a workgroup owns 64 or 32 positions instead (phase 2 then occupies two
// wavefronts or one): a 14x14 map at batch 64 has 113 tiles of 128 positions for 256 compute units,
// and a workgroup's time is the chain of its input chunks, not the chip's throughput.  Weights come straight from memory in matrix-core operand order (conv_direct.h).
// The input and the output may be channel slices of one tensor (they are in a dense block): a
// workgroup reads channels below the slice it writes, and so does every other workgroup.
#include "conv_direct.h"


namespace ens {

constexpr int DN_C = 128, DN_CO = 32, DN_MAXCIN = 2048;
template <int R>
constexpr int dn_big() { return 4 * R * 64 > 2 * R * 128 ? 4 * R * 64 : 2 * R * 128; }   // ring of four input chunks, then the middle tensor

template <int OFFSET>
__device__ __forceinline__ f32x4 dn_lds_read_f4(uint32_t addr) {
    f32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
    return v;
}
__device__ __forceinline__ void dn_tie(f32x4& v) { asm volatile("" : "+v"(v)); }
// written as an instruction so that the compiler does not order it against the asynchronous loads in flight
__device__ __forceinline__ void dn_lds_write(uint32_t addr, const u32x4& v) { asm volatile("ds_write_b128 %0, %1" ::"v"(addr), "v"(v) : "memory"); }

// argv: the argument blocks of the two convolutions, gridDim.z of each (one per member of the gang)
template <int BP, int R>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void dense_layer_bf16(const ConvArgs* __restrict__ argv, const int nb_) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int G = gridDim.z;
    const ConvArgs a1 = argv[blockIdx.z], a2 = argv[G + blockIdx.z];
    constexpr int C = DN_C;
    static_assert(BP == 32 || BP == 64 || BP == 128, "one to four wavefronts of 32 positions in phase 2");
    // phase 1: wavefronts 2 along the window rows, 2 along the channels
    constexpr int WR1 = 2, TP1 = R / (32 * WR1), TC1 = 2;
    static_assert(TP1 * 32 * WR1 == R && R % 64 == 0, "window rows split evenly");
    constexpr int XO = R / 64, WO = 2 * TC1;         // loads per thread and chunk: input rows, weight fragments
    constexpr int KK = C / 16, NST = 9 * KK, PW = R == 256 ? 6 : 8;   // phase 2: steps per tap, steps, steps the weights run ahead (registers)
    constexpr int XS = R * 64;                       // bytes of an input chunk: R rows of 32 channels
    constexpr int T1B = R * 128;                     // bytes of a 64-channel block of the middle tensor
    constexpr int BIG = dn_big<R>();

    const int W1 = a1.W + 1, H1 = a1.H + 1;
    const int PP = nb_ * H1 * W1;
    const int t = threadIdx.x, lane = t & 63, lrow = lane & 31, lhalf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int n_ptiles = (PP + BP - 1) / BP;
    int ptile, ctile;
    tile_of_block(n_ptiles, 1, &ptile, &ctile);
    const int pp0 = ptile * BP;
    const int cin1 = a1.cin;

    // LDS: x chunks, then the middle tensor | window row -> pixel index (-1: none) | biases | scales | pre-activation
    unsigned char* const big = lds;
    int* const tbl = (int*)(big + BIG);
    float* const b1l = (float*)(tbl + R);
    float* const b2l = b1l + C;
    constexpr int SBS = C + DN_CO;                   // from a channel's bias to its scale
    float* const psl = b2l + DN_CO + SBS;            // pre-activation scale of the cin input channels
    float* const phl = psl + cin1;                   // shift
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
    // Everything the tables need from memory is asked for at once (a round trip to memory is about 2000
    // clocks: one per 256 input channels, as a loop of load and store, was a quarter of the kernel at 1888 channels);
    // the window table is worked out while the answers travel.
    constexpr int NPRE = DN_MAXCIN / 256;
    float ps_r[NPRE], ph_r[NPRE];
#pragma unroll
    for (int j = 0; j < NPRE; j++) {
        const int i = t + 256 * j;
        ps_r[j] = i < cin1 ? ENS_GLOBAL(float, a1.pre_scale)[i] : 0.f;
        ph_r[j] = i < cin1 ? ENS_GLOBAL(float, a1.pre_shift)[i] : 0.f;
    }
    const float bias_r = t < C ? ENS_GLOBAL(float, a1.bias)[t] : (t < C + DN_CO ? ENS_GLOBAL(float, a2.bias)[t - C] : 0.f);
    const float scale_r = t < C ? ENS_GLOBAL(float, a1.scale)[t] : (t < C + DN_CO ? ENS_GLOBAL(float, a2.scale)[t - C] : 0.f);
    // The 3x3 filter (72 KB, the same for every workgroup) is touched once, a line per lane, so that phase 2, which
    // streams it a few steps ahead of its use, finds it in the L2 instead of waiting for memory step after step.
    float touch = 0.f;
    if (wave == 3) {
        constexpr int W2B = 9 * C * DN_CO * 2;
#pragma unroll
        for (int i = 0; i < (W2B + 8191) / 8192; i++) {
            const int off = i * 8192 + lane * 128;
            if (off < W2B) touch += ENS_GLOBAL(float, a2.wpk)[off / 4];
        }
    }
    raster_table(tbl, R, pp0 - (W1 + 1), PP, H1, W1, a1.H, a1.W);
    if (t < C + DN_CO) {                             // b1l[0..C), b2l[0..CO) lie in a row, and so do the scales SBS further on
        b1l[t] = bias_r;
        b1l[SBS + t] = scale_r;
    }
#pragma unroll
    for (int j = 0; j < NPRE; j++) {
        const int i = t + 256 * j;
        if (i < cin1) {
            psl[i] = ps_r[j];
            phl[i] = ph_r[j];
        }
    }
    asm volatile("" ::"v"(touch));                   // the touches only have to have been issued
    __syncthreads();

    // ---- load side.  Offsets past the end of a buffer give zeros in LDS (loads) or are dropped
    //      (stores); 2^31 is past the end of every buffer the launcher admits.
    constexpr unsigned OOBV = 0x80000000u;
    const unsigned npix = (unsigned)nb_ * (unsigned)(a1.H * a1.W);
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc((void*)a1.x.p, 0, (int)(npix * (unsigned)a1.x.stride * 2u), 0x00020000);
    const __amdgpu_buffer_rsrc_t w2res = __builtin_amdgcn_make_buffer_rsrc((void*)a2.wpk, 0, (int)(9u * C * DN_CO * 2u), 0x00020000);
    // thread roles in a load instruction of the workgroup (4 KB of 64-byte rows): row and swizzled chunk
    const int r4 = t >> 2, c4 = (t & 3) ^ ((r4 >> 2) & 3);
    unsigned xvo[XO];
#pragma unroll
    for (int s = 0; s < XO; s++) {
        const int p = tbl[r4 + 64 * s];
        xvo[s] = p >= 0 ? (unsigned)(p * a1.x.stride * 2) + (unsigned)(a1.x.c0 * 2 + c4 * 16) : OOBV;
    }
    unsigned char* const mine = lds + wave * 1024;               // this wave's quarter of a 4 KB load
    auto issue_x = [&](int buf, int kc) {                        // buf: place in the ring
#pragma unroll
        for (int s = 0; s < XO; s++)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (lds_ptr_t)(mine + buf * XS + s * 4096), LDS_LOAD_BYTES, xvo[s], kc * 64, 0, 0);
    };
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
    // phase 2: this wave's 32 positions; its first weight fragments are asked for before phase 1 has written its result
    const int wp0 = wave * 32;
    const unsigned wv2 = (unsigned)(lane * 16);
    bf16x8 wq2[PW];

    // ---- phase 1: the middle tensor over the window.  The input chunks come through a ring of four LDS
    //      buffers: while the matrix cores work on chunk kc (already pre-activated), the same wavefront turns
    //      its own pieces of chunk kc + 1 into relu(x * scale + shift) in place, and chunks kc + 2 and kc + 3
    //      are on their way; the weights of chunk kc + 2 are asked for while chunk kc is used.  Loads complete
    //      in the order they were issued, so a wait counts what was issued after the load it needs.
    {
        const int xr = row0 + lrow;
        const uint32_t psl0 = (uint32_t)(uintptr_t)(lds_ptr_t)psl;
        const uint32_t xs1 = lds0 + (uint32_t)(xr * 64 + ((lhalf ^ ((xr >> 2) & 3)) << 4));
        const uint32_t own0 = lds0 + (uint32_t)(wave * 1024 + lane * 16);   // where this thread's piece of a 4 KB load lands
        f32x16 acc[TC1][TP1];
#pragma unroll
        for (int i = 0; i < TC1; i++)
#pragma unroll
            for (int j = 0; j < TP1; j++) bn_zero(acc[i][j]);
        issue_x(0, 0);
        if (nk1 > 1) issue_x(1, 1);
        if (nk1 > 2) issue_x(2, 2);
        // a * XO + b * WO loads may still be in flight (fewer than allowed is always safe)
        auto wait_vm = [&](int a, int b) {
            if (a == 2 && b == 2) bn_wait_vm<2 * XO + 2 * WO>();
            else if (a == 2 && b == 1) bn_wait_vm<2 * XO + WO>();
            else if (a == 1 && b == 2) bn_wait_vm<XO + 2 * WO>();
            else if (a == 2 && b == 0) bn_wait_vm<2 * XO>();
            else if (a == 1 && b == 0) bn_wait_vm<XO>();
            else if (a == 0 && b == 1) bn_wait_vm<WO>();
            else bn_wait_vm<0>();
        };
        // The pre-activation, in place: every thread converts the 16-byte pieces its own loads brought in (the
        // same 8 channels of XO rows).  Applied to the fragments on their way to the matrix cores instead, each
        // value would be converted by both wavefronts that share its rows.
        bf16x8 xv[XO];
        f32x4 ps0, ps1, ph0, ph1;
        auto pre_read = [&](int kc) {
            const uint32_t pa = psl0 + (uint32_t)((kc * 32 + 8 * c4) * 4), ha = pa + (uint32_t)(cin1 * 4);
            ps0 = dn_lds_read_f4<0>(pa); ps1 = dn_lds_read_f4<16>(pa);
            ph0 = dn_lds_read_f4<0>(ha); ph1 = dn_lds_read_f4<16>(ha);
            const uint32_t own = own0 + (uint32_t)((kc & 3) * XS);
            bn_unroll<XO>([&](auto sc) { xv[decltype(sc)::value] = bn_lds_read<decltype(sc)::value * 4096>(own); });
        };
        auto pre_tie = [&]() {
            dn_tie(ps0); dn_tie(ps1); dn_tie(ph0); dn_tie(ph1);
#pragma unroll
            for (int x = 0; x < XO; x++) bn_tie(xv[x]);
        };
        auto pre_math = [&]() {
            const float sc[8] = {ps0[0], ps0[1], ps0[2], ps0[3], ps1[0], ps1[1], ps1[2], ps1[3]};
            const float sh[8] = {ph0[0], ph0[1], ph0[2], ph0[3], ph1[0], ph1[1], ph1[2], ph1[3]};
#pragma unroll
            for (int x = 0; x < XO; x++) {
                u32x4 u = __builtin_bit_cast(u32x4, xv[x]);
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const float lo = __uint_as_float(u[q] << 16), hi = __uint_as_float(u[q] & 0xFFFF0000u);
                    typedef short s16x2 __attribute__((ext_vector_type(2)));
                    const s16x2 z = {0, 0};                      // relu on the rounded pair: a negative bf16 is a negative 16-bit integer
                    u[q] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(
                        __builtin_bit_cast(s16x2, pack_bf16x2(fmaf(lo, sc[2 * q], sh[2 * q]), fmaf(hi, sc[2 * q + 1], sh[2 * q + 1]))), z));
                }
                xv[x] = __builtin_bit_cast(bf16x8, u);
            }
        };
        auto pre_write = [&](int kc) {
            const uint32_t own = own0 + (uint32_t)((kc & 3) * XS);
#pragma unroll
            for (int x = 0; x < XO; x++) dn_lds_write(own + (uint32_t)(x * 4096), __builtin_bit_cast(u32x4, xv[x]));
        };
        // chunk 0 is converted before the loop
        wait_vm((nk1 > 1) + (nk1 > 2), 0);
        pre_read(0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        pre_tie();
        pre_math();
        pre_write(0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        // One chunk: `wc` holds its weights, `wl` receives those of chunk kc + 2.  The roles of the three weight
        // sets rotate with period three, so the loop below is written out three chunks at a time: a rotation
        // through register copies would have to wait for the loads just issued.
        // `steady`: chunk kc + 3 exists, so every load is issued and the wait is one constant (with
        // conditional loads in the loop the compiler's own waits for the weight registers assume the path
        // on which nothing was issued, and wait for everything).
        auto chunk = [&](auto mode_c, bf16x8 (&wc)[2][TC1], bf16x8 (&wl)[2][TC1], const int kc) {
            constexpr bool steady = decltype(mode_c)::value > 0, first = decltype(mode_c)::value == 2;
            // behind the barrier: chunk kc is converted, nobody reads chunk kc - 1 any more
            if (steady || kc + 3 < nk1) issue_x((kc + 3) & 3, kc + 3);
            if (steady || kc + 2 < nk1) load_w(wl, kc + 2);
            const uint32_t xs = xs1 + (uint32_t)((kc & 3) * XS);
            bf16x8 xf[2][TP1];
            bn_unroll<TP1>([&](auto j) { xf[0][decltype(j)::value] = bn_lds_read<decltype(j)::value * 2048>(xs); });
            bn_unroll<TP1>([&](auto j) { xf[1][decltype(j)::value] = bn_lds_read<decltype(j)::value * 2048>(xs ^ 32u); });
            // the loads of chunk kc + 1 have landed: issued after them are the loads of chunks kc + 2 and kc + 3
            // and the weights of chunks kc + 1 (from chunk 1 on: the first two sets are asked for up front) and kc + 2
            if (first) bn_wait_vm<2 * XO + WO>();
            else if (steady) bn_wait_vm<2 * XO + 2 * WO>();
            else wait_vm((kc + 2 < nk1) + (kc + 3 < nk1), (kc + 2 < nk1) + (kc >= 1 && kc + 1 < nk1));
            const int kn = steady || kc + 1 < nk1 ? kc + 1 : kc; // after the last chunk: converted again, not written
            pre_read(kn);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int ks = 0; ks < 2; ks++)
#pragma unroll
                for (int j = 0; j < TP1; j++) bn_tie(xf[ks][j]);
            pre_tie();
            // matrix-core work on chunk kc and vector work on chunk kc + 1, independent of each other
#pragma unroll
            for (int ks = 0; ks < 2; ks++)
#pragma unroll
                for (int i = 0; i < TC1; i++)
#pragma unroll
                    for (int j = 0; j < TP1; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wc[ks][i], xf[ks][j], acc[i][j], 0, 0, 0);
            pre_math();
            if (steady || kc + 1 < nk1) pre_write(kn);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
        };
        constexpr std::integral_constant<int, 0> near_the_end{};
        constexpr std::integral_constant<int, 1> all_there{};
        constexpr std::integral_constant<int, 2> all_there_first{};  // chunk 0: the weights of chunk 1 were asked for up front
        int kc = 0;
        if (nk1 > 5) {                                           // chunks 0 to 2 of a long input: the same code as the loop's
            chunk(all_there_first, w0, w2, 0);
            chunk(all_there, w1, w0, 1);
            chunk(all_there, w2, w1, 2);
            kc = 3;
        }
        for (; kc + 5 < nk1; kc += 3) {
            chunk(all_there, w0, w2, kc);
            chunk(all_there, w1, w0, kc + 1);
            chunk(all_there, w2, w1, kc + 2);
        }
        for (; kc < nk1; kc += 3) {
            chunk(near_the_end, w0, w2, kc);
            if (kc + 1 < nk1) chunk(near_the_end, w1, w0, kc + 1);
            if (kc + 2 < nk1) chunk(near_the_end, w2, w1, kc + 2);
        }
        if (wave < BP / 32) {                                    // the wavefronts that take part in phase 2
#pragma unroll
            for (int s = 0; s < PW; s++) wq2[s] = bn_wload(w2res, wv2, s * 1024);
        }
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

    // ---- phase 2: the nine taps over the middle tensor, 32 output channels; no barrier, weights PW steps ahead
    __syncthreads();                                             // the middle tensor is complete
    if (wave < BP / 32) {
        const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc((void*)a2.y.p, 0, (int)(npix * (unsigned)a2.y.stride * 2u), 0x00020000);
        const int pout = tbl[W1 + 1 + wp0 + lrow];               // the centre tap's rows: this tile's outputs
        const unsigned yo = pout >= 0 ? (unsigned)(pout * a2.y.stride * 2) + (unsigned)((a2.y.c0 + 8 * lhalf) * 2) : OOBV;
        f32x16 acc;
        bn_zero(acc);
        uint32_t xoff[9];                                        // tap (dh, dw): dh rows of the padded raster down, dw positions right
#pragma unroll
        for (int tap = 0; tap < 9; tap++) {
            const uint32_t q = (uint32_t)(wp0 + lrow + (tap / 3) * W1 + tap % 3);
            xoff[tap] = lds0 + q * 128 + ((((uint32_t)lhalf) ^ ((q >> 1) & 7)) << 4);
        }
        bf16x8 xf[2];
        auto read_frag = [&](auto st_c, auto b_c) {
            constexpr int st = decltype(st_c)::value, b = decltype(b_c)::value;
            constexpr int tap = st / KK, kk = st % KK;           // step kk of the tap: block kk / 4 of the middle tensor, chunks 2 (kk % 4) and + 1
            xf[b] = bn_lds_read<0>((xoff[tap] + (uint32_t)((kk / 4) * T1B)) ^ (uint32_t)((kk % 4) << 5));
        };
        read_frag(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        bn_unroll<NST>([&](auto st_c) {
            constexpr int st = decltype(st_c)::value, b = st & 1, slot = st % PW;
            if constexpr (st + 1 < NST) {
                read_frag(std::integral_constant<int, st + 1>{}, std::integral_constant<int, b ^ 1>{});
                asm volatile("s_waitcnt lgkmcnt(1)" ::: "memory");
            } else {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
            bn_tie(xf[b]);
            const bf16x8 wc = wq2[slot];
            if constexpr (st + PW < NST) wq2[slot] = bn_wload(w2res, wv2, (st + PW) * 1024);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wc, xf[b], acc, 0, 0, 0);
        });
        // register v of a lane is channel 16(v/8) + 8(lane/32) + v%8 of its position; stores to positions
        // without a pixel carry the out-of-range offset and are dropped by the hardware
#pragma unroll
        for (int k = 0; k < 2; k++) __builtin_amdgcn_raw_buffer_store_b128(bn_pack(acc, k, a2.act, b2l + 8 * lhalf, SBS), yres, yo, 32 * k, 0);
    }
}

// ---- host side -----------------------------------------------------------------------------
constexpr int DENSE_LDS_LIMIT = 160 * 1024;
constexpr int DENSE_MIN_TILES = 1;   // measured on a DenseNet-121-shaped member: the one kernel is faster at every batch size, 1 to 128

struct DensePlan { int bp, rows; size_t bytes; int tiles; };

static bool dense_plan(const ConvArgs& a1, const ConvArgs& a2, int nb, int G, DensePlan* pl) {
    if (a1.kh != 1 || a1.kw != 1 || a1.sh != 1 || a1.sw != 1 || a1.pt != 0 || a1.pl != 0 || a1.Ho != a1.H || a1.Wo != a1.W) return false;
    if (!a1.pre_scale || !a1.pre_shift || a1.res.p || a2.res.p || a2.pre_scale) return false;
    if (a2.kh != 3 || a2.kw != 3 || a2.sh != 1 || a2.sw != 1 || a2.pt != 1 || a2.pl != 1) return false;
    if (a2.H != a1.H || a2.W != a1.W || a2.Ho != a1.H || a2.Wo != a1.W) return false;
    if (a1.cout != DN_C || a2.cin != DN_C || a2.cout != DN_CO || a1.cin % 32 || a1.cin > DN_MAXCIN || !a1.wpk || !a2.wpk) return false;
    // the middle tensor is skipped: the 3x3 reads what the first convolution writes
    if (a2.x.p != a1.y.p || a2.x.c0 != a1.y.c0) return false;
    // input and output may share a tensor when the output slice lies past the input's channels
    if (a2.y.p == a1.x.p && a2.y.c0 < a1.x.c0 + a1.cin) return false;
    // 32-bit byte offsets with 2^31 standing for 'outside'; float index arithmetic is exact below 2^24
    const long long P = (long long)nb * a1.H * a1.W;
    if (P * a1.x.stride * 2 >= 0x7FFFFF00LL || P * a2.y.stride * 2 >= 0x7FFFFF00LL) return false;
    const long long PP = (long long)nb * (a1.H + 1) * (a1.W + 1);
    if (PP >= (1LL << 24)) return false;
    if (a1.x.stride % 8 || a1.x.c0 % 8 || a2.y.stride % 8 || a2.y.c0 % 8) return false;
    // positions per workgroup: 128, or fewer while that does not give every compute unit a workgroup
    // and the window of the smaller tile fits the next smaller number of rows
    const int reach = 2 * (a1.W + 1) + 2;
    pl->bp = 128;
    if (G * ((PP + 127) / 128) < cu_budget() && 64 + reach <= 128) pl->bp = 64;
    if (G * ((PP + 63) / 64) < cu_budget() && 32 + reach <= 64) pl->bp = 32;
    const int need = pl->bp + reach;
    pl->rows = pl->bp == 32 ? 64 : pl->bp == 64 ? 128 : need <= 192 ? 192 : 256;
    if (need > pl->rows) return false;
    const int big = pl->rows == 64 ? dn_big<64>() : pl->rows == 128 ? dn_big<128>() : pl->rows == 192 ? dn_big<192>() : dn_big<256>();
    pl->bytes = (size_t)big + (size_t)pl->rows * 4 + (size_t)(2 * (DN_C + DN_CO) + 2 * a1.cin) * 4;
    pl->tiles = (int)((PP + pl->bp - 1) / pl->bp);
    return 2 * pl->bytes <= (size_t)DENSE_LDS_LIMIT;
}

bool conv_dense_applicable(const ConvArgs& a1, const ConvArgs& a2, int nb, int G) {
    DensePlan pl;
    if (!dense_plan(a1, a2, nb, G, &pl)) return false;
    long long least = DENSE_MIN_TILES;
    return (long long)pl.tiles * G >= least;
}

const char* conv_dense_name() { return "dense_layer_bf16"; }

template <int BP, int R>
static hipError_t launch_dense_variant(const ConvArgs* argv, int G, int nb, const DensePlan& pl, hipStream_t s) {
    static bool raised = false;                                  // LDS above 64 KB has to be asked for once
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void*)&dense_layer_bf16<BP, R>, hipFuncAttributeMaxDynamicSharedMemorySize, DENSE_LDS_LIMIT);
        if (e != hipSuccess) return e;
        raised = true;
    }
    ENS_LAUNCH((dense_layer_bf16<BP, R>), dim3((unsigned)pl.tiles, 1, G), dim3(256), pl.bytes, s, argv, nb);
    return hipGetLastError();
}

hipError_t launch_conv_dense(const ConvArgs& a1, const ConvArgs& a2, const ConvArgs* argv, int G, int nb, hipStream_t s) {
    DensePlan pl;
    if (!dense_plan(a1, a2, nb, G, &pl)) return hipErrorInvalidValue;
    if (pl.bp == 32) return launch_dense_variant<32, 64>(argv, G, nb, pl, s);
    if (pl.bp == 64) return launch_dense_variant<64, 128>(argv, G, nb, pl, s);
    return pl.rows == 192 ? launch_dense_variant<128, 192>(argv, G, nb, pl, s) : launch_dense_variant<128, 256>(argv, G, nb, pl, s);
}

}  // namespace ens
