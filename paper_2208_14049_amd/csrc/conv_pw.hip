// 1x1 convolution (stride 1, or a stride without padding: the shortcuts of residual stages) on the CDNA4 matrix cores with the weights taken straight from memory
// in matrix-core operand order (conv_direct.h): the 1x1 layers of residual bottlenecks that do not
// run inside the fused bottleneck kernel, the expansion and projection layers of inverted-residual
// blocks, the pointwise halves of separable convolutions.  Channel counts are multiples of 8; the
// operand-ordered copy of the weights is padded with zeros to 32 rows and 64 columns.
//
// GEMM view: rows = pixels, columns = output channels, K = input channels.  A workgroup of four
// wavefronts owns 128 pixels x BC channels.  The pixels' input arrives 64 channels at a time
// through a three-deep ring of LDS buffers filled by asynchronous global-to-LDS loads, two chunks
// ahead of its use, with counted waits (loads complete in the order they were issued, so the wait
// before a chunk is used names the number of loads issued after it).  A wavefront's weight
// fragments, 1 KB in a row each, go from memory to registers two chunks ahead as well; nothing but
// the pixel fragments is read from LDS, and the one barrier per chunk covers 16 or 8 matrix-core
// instructions per wavefront where the generic kernel's covers 4 to 8 and also waits for its
// weights.  The output leaves from the accumulators as 16-byte runs of 8 channels after the
// per-channel scale and bias (which wait in LDS); the residual is asked for before the loop.
//
// Wavefront roles: WPX along the pixels, 4 / WPX along blocks of 32 channels.  WPX = 1: a wavefront
// has all 128 pixels of 32 channels (a weight fragment serves four matrix-core instructions and is
// fetched by one wavefront only), BC = 128; WPX = 2 for layers with 64 output channels or fewer.
#include "conv_direct.h"


namespace ens {

constexpr int PW_BP = 128, PW_NXB = 3, PW_XS = PW_BP * 128;

// GATE: the input is multiplied by a gate per (image, input channel) in LDS, each chunk in place by the threads
// that brought it in, before the matrix cores read it
// (the rescaling of a squeeze-excite block folded into the projection that follows it): product in fp32,
// rounded to bf16 as the separate rescaling kernel would have stored it.  The gates of the images a tile
// touches wait in LDS behind the ring, gimg images of nk * 64 floats.
template <int WPX, bool GATE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void conv1x1_direct_bf16(const ConvArgs* __restrict__ argv,
                                                                                                     const int nb_, const int gimg) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const ConvArgs a = argv[blockIdx.z];
    static_assert(WPX == 1 || WPX == 2, "one or two wavefronts along the pixels");
    constexpr int BP = PW_BP, WCG = 4 / WPX, TP = BP / (32 * WPX), BC = 32 * WCG, XS = PW_XS;
    constexpr int XO = BP / 32, WO = 4;              // loads per thread and chunk: input rows, weight fragments
    const int P = nb_ * a.Ho * a.Wo;                 // output pixels (the input's too, unless the layer has a stride)
    const int t = threadIdx.x, lane = t & 63, lrow = lane & 31, lhalf = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int n_ptiles = (P + BP - 1) / BP, n_ctiles = (a.cout + BC - 1) / BC;
    int ptile, ctile;
    tile_of_block(n_ptiles, n_ctiles, &ptile, &ctile);
    if (ptile >= n_ptiles) return;
    const int p0 = ptile * BP, c0 = ctile * BC;
    const int wp0 = (wave % WPX) * (TP * 32);
    const int wc = c0 + (wave / WPX) * 32;           // this wave's 32 channels; the last block of a layer may hold fewer
    const bool wave_ok = wc < a.cout;
    const int nk = (a.cin + 63) / 64, NS = nk * 4;   // input chunks; matrix-core steps per block of weight rows

    // Offsets past the end of a buffer give zeros (loads) or are dropped (stores); 2^31 is past the
    // end of every buffer the launcher admits.
    constexpr unsigned OOBV = 0x80000000u;
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.wpk, 0, (int)((unsigned)((a.cout + 31) / 32 * 32) * (unsigned)(nk * 64) * 2u), 0x00020000);
    const unsigned wv = wave_ok ? (unsigned)((wc / 32) * NS * 1024 + lane * 16) : OOBV;
    bf16x8 w0[4], w1[4], w2[4];                      // weights of this chunk, the next, the one after
    auto load_w = [&](bf16x8 (&w)[4], int kc) {
#pragma unroll
        for (int ks = 0; ks < 4; ks++) w[ks] = bn_wload(wres, wv, (kc * 4 + ks) * 1024);
    };
    load_w(w0, 0);
    if (nk > 1) load_w(w1, 1);

    // ---- what the epilogue needs from memory: asked for now, older than every input chunk
    const unsigned npix = (unsigned)P;
    const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc((void*)a.y.p, 0, (int)(npix * (unsigned)a.y.stride * 2u), 0x00020000);
    const bool has_res = a.res.p != nullptr;
    const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(has_res ? a.res.p : a.y.p), 0, (int)(npix * (unsigned)(has_res ? a.res.stride : a.y.stride) * 2u), 0x00020000);
    // this lane's two runs of 8 channels, wc + 8 (lane / 32) + 16 k: each exists as a whole or not at all
    const int ch0 = wc + 8 * lhalf;
    const bool run_ok[2] = {ch0 < a.cout, ch0 + 16 < a.cout};
    unsigned yo[TP][2], ro[TP][2];
#pragma unroll
    for (int j = 0; j < TP; j++) {
        const int p = p0 + wp0 + 32 * j + lrow;
#pragma unroll
        for (int k = 0; k < 2; k++) {
            const bool ok = p < P && run_ok[k];
            yo[j][k] = ok ? (unsigned)(p * a.y.stride * 2) + (unsigned)((a.y.c0 + ch0) * 2) : OOBV;
            ro[j][k] = ok ? (unsigned)(p * a.res.stride * 2) + (unsigned)((a.res.c0 + ch0) * 2) : OOBV;
        }
    }
    u32x4 res[TP][2];
    if (has_res) {
#pragma unroll
        for (int j = 0; j < TP; j++) {
            res[j][0] = __builtin_amdgcn_raw_buffer_load_b128(rres, ro[j][0], 0, 0);
            res[j][1] = __builtin_amdgcn_raw_buffer_load_b128(rres, ro[j][1], 32, 0);
        }
    }
    f32x16 acc[TP];
#pragma unroll
    for (int j = 0; j < TP; j++) bn_zero(acc[j]);
    // bias and scale of the tile's BC channels wait in LDS behind the ring (zeros and ones past the last
    // channel).  They are asked for here and stored once the first input chunks are on their way: a store
    // right here would hold those back by a round trip to memory.
    float* const sbl = (float*)(lds + PW_NXB * XS);
    const bool sb_ok = t < BC && c0 + t < a.cout;
    const float bias_r = sb_ok ? ENS_GLOBAL(float, a.bias)[c0 + t] : 0.f;
    const float scale_r = sb_ok ? ENS_GLOBAL(float, a.scale)[c0 + t] : 1.f;
    float* const gl = sbl + 2 * 128;                 // GATE: [image of the tile][nk * 64] gates, zeros past the last channel
    int gpiece[BP / 32];                             // GATE: first gate of the 16 bytes this thread brings in of input row r8 + 32 s, less the chunk's offset
    const int HW = a.H * a.W, cinp = nk * 64;
    const int n_first = p0 / HW, n_last = min(p0 + BP - 1, P - 1) / HW;

    // ---- input chunks: thread t fills chunk slot t % 8 of rows t / 8 + 32 s with the swizzled chunk
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.x.p, 0, (int)((unsigned)nb_ * (unsigned)(a.H * a.W) * (unsigned)a.x.stride * 2u), 0x00020000);
    const int r8 = t >> 3, c8 = (t & 7) ^ ((r8 >> 1) & 7);
    const bool strided = a.sh != 1 || a.sw != 1;
    if constexpr (GATE) {
#pragma unroll
        for (int s = 0; s < XO; s++) gpiece[s] = (min(p0 + r8 + 32 * s, P - 1) / HW - n_first) * cinp + 8 * c8;
    }
    unsigned xvo[XO];
#pragma unroll
    for (int s = 0; s < XO; s++) {
        const int p = p0 + r8 + 32 * s;
        int pin = p;                                 // the input pixel of output pixel p
        if (strided && p < P) {
            // p -> (image, row, column) with one double multiply per division and a correction step
            int n = (int)((double)p * a.inv_hw);
            int rem = p - n * (a.Ho * a.Wo);
            if (rem < 0) { n--; rem += a.Ho * a.Wo; } else if (rem >= a.Ho * a.Wo) { n++; rem -= a.Ho * a.Wo; }
            int ho = (int)((double)rem * a.inv_w);
            int wo = rem - ho * a.Wo;
            if (wo < 0) { ho--; wo += a.Wo; } else if (wo >= a.Wo) { ho++; wo -= a.Wo; }
            pin = (n * a.H + ho * a.sh) * a.W + wo * a.sw;
        }
        xvo[s] = p < P ? (unsigned)(pin * a.x.stride * 2) + (unsigned)(a.x.c0 * 2 + c8 * 16) : OOBV;
    }
    // in the last chunk of a layer whose input channels are not a multiple of 64 this thread's 8 channels
    // may lie past the last one: zeros then (what follows them in memory belongs to the next pixel)
    const bool tail_ok = (nk - 1) * 64 + c8 * 8 < a.cin;
    unsigned char* const mine = lds + wave * 1024;               // this wave's quarter of a 4 KB load
    auto issue_x = [&](int buf, int kc) {
        const bool live = kc + 1 < nk || tail_ok;
#pragma unroll
        for (int s = 0; s < XO; s++)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (lds_ptr_t)(mine + buf * XS + s * 4096), LDS_LOAD_BYTES, live ? xvo[s] : OOBV,
                                                     kc * 128, 0, 0);
    };
    issue_x(0, 0);
    if (nk > 1) issue_x(1, 1);
    // the first barrier of the chunk loop comes between these writes and their readers
    if (t < BC) {
        sbl[t] = bias_r;
        sbl[BC + t] = scale_r;
    }
    if constexpr (GATE) {
        // the gates of the tile's images, sixteen loads in flight per thread (one at a time, the table of a
        // 2688-channel layer over four images was forty round trips to memory)
        const int n_g = gimg * cinp;
        for (int i0 = t; i0 < n_g; i0 += 256 * 16) {
            float g[16];
#pragma unroll
            for (int u = 0; u < 16; u++) {
                const int i = i0 + 256 * u;
                const int img = i / cinp, c = i - img * cinp;
                g[u] = (i < n_g && c < a.cin && n_first + img <= n_last) ? ENS_GLOBAL(float, a.gate)[(long long)(n_first + img) * a.gate_stride + c] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 16; u++)
                if (i0 + 256 * u < n_g) gl[i0 + 256 * u] = g[u];
        }
        __syncthreads();                                         // the first chunk is gated before the loop's first barrier
    }

    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
    const int xr = wp0 + lrow;
    const uint32_t xs0 = lds0 + (uint32_t)(xr * 128 + ((lhalf ^ ((xr >> 1) & 7)) << 4));
    // One chunk: `wc` holds its weights, `wl` receives those of chunk kc + 2, BUF is its place in the
    // ring.  The three roles rotate with period three, so the loop below is written out three chunks at
    // a time: a rotation through register copies would have to wait for the loads just issued.
    auto chunk = [&](auto buf_c, bf16x8 (&wc_)[4], bf16x8 (&wl)[4], const int kc) {
        constexpr int buf = decltype(buf_c)::value;
        // chunk kc has landed (this wave's part; with the barrier everybody's), and nobody still reads
        // the buffer that chunk kc + 2 goes to.  Issued after chunk kc: the weights and the input of
        // chunk kc + 1 (chunk 0: only the input of chunk 1, the weights went first).
        if (kc == 0) {
            if (nk > 1) bn_wait_vm<XO>(); else bn_wait_vm<0>();
        } else {
            if (kc + 1 < nk) bn_wait_vm<WO + XO>(); else bn_wait_vm<0>();
        }
        if constexpr (GATE) {
            // every thread multiplies the 16-byte pieces it brought in itself by their gates, in place and once per value
            // (done per fragment, each wavefront along the output channels did it again: twenty vector instructions for
            // every matrix-core instruction); the barrier below hands the gated chunk to the readers
            unsigned char* const my = mine + buf * XS + lane * 16;
            u32x4 xp[XO];
            f32x4 g0[XO], g1[XO];
#pragma unroll
            for (int s2 = 0; s2 < XO; s2++) {
                xp[s2] = *(const u32x4*)(my + s2 * 4096);
                const float* gp = gl + gpiece[s2] + kc * 64;
                g0[s2] = *(const f32x4*)gp;
                g1[s2] = *(const f32x4*)(gp + 4);
            }
#pragma unroll
            for (int s2 = 0; s2 < XO; s2++) {
                u32x4 u = xp[s2];
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const float lo = __uint_as_float(u[q] << 16), hi = __uint_as_float(u[q] & 0xFFFF0000u);
                    const float gq0 = q < 2 ? g0[s2][2 * q] : g1[s2][2 * q - 4], gq1 = q < 2 ? g0[s2][2 * q + 1] : g1[s2][2 * q - 3];
                    u[q] = pack_bf16x2(lo * gq0, hi * gq1);
                }
                *(u32x4*)(my + s2 * 4096) = u;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        __builtin_amdgcn_s_barrier();
        if (kc + 2 < nk) {
            load_w(wl, kc + 2);
            issue_x((buf + 2) % 3, kc + 2);
        }
        const uint32_t xs = xs0 + (uint32_t)(buf * XS);
        bf16x8 xf[2][TP];
        auto read_frags = [&](auto ks_c, auto b_c) {
            constexpr int ks = decltype(ks_c)::value, b = decltype(b_c)::value;
            const uint32_t xa = xs ^ (uint32_t)(ks << 5);
            bn_unroll<TP>([&](auto j) { xf[b][decltype(j)::value] = bn_lds_read<decltype(j)::value * 4096>(xa); });
        };
        read_frags(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        bn_unroll<4>([&](auto ks_c) {
            constexpr int ks = decltype(ks_c)::value, b = ks & 1;
            // the next step's reads are issued first; LDS returns in order, so once no more than those
            // are outstanding this step's fragments are complete
            if constexpr (ks + 1 < 4) {
                read_frags(std::integral_constant<int, ks + 1>{}, std::integral_constant<int, b ^ 1>{});
                asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(TP) : "memory");
            } else {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
#pragma unroll
            for (int j = 0; j < TP; j++) bn_tie(xf[b][j]);
#pragma unroll
            for (int j = 0; j < TP; j++) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wc_[ks], xf[b][j], acc[j], 0, 0, 0);
        });
    };
    int kc = 0;
    for (; kc + 2 < nk; kc += 3) {
        chunk(std::integral_constant<int, 0>{}, w0, w2, kc);
        chunk(std::integral_constant<int, 1>{}, w1, w0, kc + 1);
        chunk(std::integral_constant<int, 2>{}, w2, w1, kc + 2);
    }
    if (kc < nk) chunk(std::integral_constant<int, 0>{}, w0, w2, kc);
    if (kc + 1 < nk) chunk(std::integral_constant<int, 1>{}, w1, w0, kc + 1);

    // ---- output: register v of a lane is channel wc + 16(v/8) + 8(lane/32) + v%8 of its pixel.  Stores
    //      to rows past the last pixel carry the out-of-range offset and are dropped by the hardware.
#pragma unroll
    for (int j = 0; j < TP; j++)
#pragma unroll
        for (int k = 0; k < 2; k++) {
            const float* sb = sbl + (ch0 - c0);
            const u32x4 o = has_res ? bn_pack_res<true>(acc[j], k, res[j][k], a.act, sb, BC) : bn_pack_res<false>(acc[j], k, res[j][k], a.act, sb, BC);
            __builtin_amdgcn_raw_buffer_store_b128(o, yres, yo[j][k], 32 * k, 0);
        }
}

// ---- host side -----------------------------------------------------------------------------
static bool pw_shape_ok(const ConvArgs& a, int nb) {
    if (a.kh != 1 || a.kw != 1 || a.pt != 0 || a.pl != 0 || a.sh < 1 || a.sw < 1) return false;
    if (a.Ho != (a.H - 1) / a.sh + 1 || a.Wo != (a.W - 1) / a.sw + 1) return false;
    if ((a.sh != 1 || a.sw != 1) && a.gate) return false;       // the gates are looked up by the input's image, which a tile finds from its output pixels
    if (a.pre_scale || !a.wpk || a.cin % 8 || a.cout % 8) return false;
    // 32-bit byte offsets with 2^31 standing for 'outside'
    const long long P = (long long)nb * a.Ho * a.Wo, Pin = (long long)nb * a.H * a.W;
    if (Pin * a.x.stride * 2 >= 0x7FFFFF00LL || P * a.y.stride * 2 >= 0x7FFFFF00LL) return false;
    if (a.res.p && P * a.res.stride * 2 >= 0x7FFFFF00LL) return false;
    if ((long long)(a.cout + 31) * (a.cin + 63) * 2 >= 0x7FFFFF00LL) return false;
    if (a.x.stride % 8 || a.x.c0 % 8 || a.y.stride % 8 || a.y.c0 % 8) return false;
    if (a.res.p && (a.res.stride % 8 || a.res.c0 % 8)) return false;
    return true;
}

// GATE: images a tile of PW_BP pixels can touch, and the bytes of their gates in LDS
static int pw_gate_images(const ConvArgs& a) { return (PW_BP - 1) / (a.H * a.W) + 2; }
static size_t pw_gate_bytes(const ConvArgs& a) { return a.gate ? (size_t)pw_gate_images(a) * ((a.cin + 63) / 64 * 64) * sizeof(float) : 0; }
constexpr size_t PW_LDS_BASE = (size_t)PW_NXB * PW_XS + 2 * 128 * sizeof(float);

bool conv_pw_applicable(const ConvArgs& a, int nb, int G) {
    // (small maps with thousands of channels leave room for one workgroup per compute unit only: still better than a pass more)
    if (a.gate && (a.gate_stride < a.cin || PW_LDS_BASE + pw_gate_bytes(a) > 160 * 1024)) return false;
    return pw_shape_ok(a, nb);
}



template <int WPX, bool GATE>
static hipError_t launch_pw_variant(const ConvArgs& a, const ConvArgs* argv, int G, int nb, hipStream_t s) {
    constexpr int BC = 32 * (4 / WPX);
    const long long P = (long long)nb * a.Ho * a.Wo;
    const dim3 grid((unsigned)(((P + PW_BP - 1) / PW_BP) * ((a.cout + BC - 1) / BC)), 1, G);
    const size_t bytes = PW_LDS_BASE + pw_gate_bytes(a);
    if (bytes > 64 * 1024) {                                     // LDS above 64 KB has to be asked for once
        static bool raised = false;
        if (!raised) {
            hipError_t e = hipFuncSetAttribute((const void*)&conv1x1_direct_bf16<WPX, GATE>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
            raised = true;
        }
    }
    ENS_LAUNCH((conv1x1_direct_bf16<WPX, GATE>), grid, dim3(256), bytes, s, argv, nb, GATE ? pw_gate_images(a) : 0);
    return hipGetLastError();
}

// 128 x 128 tiles unless the layer has 64 output channels or fewer, or so few pixels that those tiles
// number fewer than the compute units (measured over the 1x1 layers of a ResNet-50 at batches of 16 to
// 128: with 196 tiles or fewer the 128 x 64 tile is faster or equal, with 392 or more the larger one)
static int pw_wpx(const ConvArgs& a, int nb, int G) {
    const long long tiles = (((long long)nb * a.Ho * a.Wo + PW_BP - 1) / PW_BP) * ((a.cout + 127) / 128) * G;
    int wpx = a.cout <= 64 || tiles < cu_budget() ? 2 : 1;
    return wpx;
}

const char* conv_pw_name(const ConvArgs& a, int G) {
    if (a.gate) return pw_wpx(a, a.nb, G) == 2 ? "conv1x1_direct_bf16<128x64,gate>" : "conv1x1_direct_bf16<128x128,gate>";
    return pw_wpx(a, a.nb, G) == 2 ? "conv1x1_direct_bf16<128x64>" : "conv1x1_direct_bf16<128x128>";
}

hipError_t launch_conv_pw(const ConvArgs& a, const ConvArgs* argv, int G, int nb, hipStream_t s) {
    if (!pw_shape_ok(a, nb)) return hipErrorInvalidValue;
    if (a.gate) {
        if (!conv_pw_applicable(a, nb, G)) return hipErrorInvalidValue;
        return pw_wpx(a, nb, G) == 2 ? launch_pw_variant<2, true>(a, argv, G, nb, s) : launch_pw_variant<1, true>(a, argv, G, nb, s);
    }
    return pw_wpx(a, nb, G) == 2 ? launch_pw_variant<2, false>(a, argv, G, nb, s) : launch_pw_variant<1, false>(a, argv, G, nb, s);
}

}  // namespace ens
