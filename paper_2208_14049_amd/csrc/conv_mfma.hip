// Implicit-GEMM convolution on the CDNA4 matrix cores (gfx950), bf16 in, fp32 accumulate.
//
// GEMM view of a convolution over NHWC activations:
//   rows    P = nb*Ho*Wo output pixels
//   columns cout output channels
//   depth   K = kh*kw*cin, input channel fastest, so 8 consecutive k are 16 contiguous bytes
//           both in the activation tensor (one pixel, one tap) and in the [cout][K] weights.
//
// A workgroup of 4 wavefronts computes a BP x BC tile of the output.  The K loop walks tiles of 64
// through a ring of NS LDS stages that is filled by asynchronous global-to-LDS loads
// (global_load_lds_dwordx4): a lane names a 16-byte chunk in global memory and the hardware drops
// it at "stage base + lane * 16" in LDS without passing through registers, so NS-1 tiles are in
// flight per workgroup while the matrix cores work on the oldest one.  What a load must not read
// (padding taps, rows past the end of the tensor, K tail) is redirected to a block of zeros.
//
// LDS layout: one 128-byte row per pixel / output channel and K tile; the 16-byte chunk c of row
// r sits in slot c ^ ((r >> 1) & 7), so that the 16 rows a quarter-wavefront reads for one
// matrix-core fragment cover all 64 banks.  Because the hardware fixes a lane's LDS slot, the
// swizzle is applied on the global side: the lane in slot s of row r fetches chunk s ^ key(r).
// A thread serves rows r0 + 32*i (r0 = thread / 8), for which key(r) is the same: one chunk
// column, hence one filter tap, per thread and K tile.
//
// The weights are the A operand of v_mfma_f32_32x32x16_bf16 and the pixels the B operand.  The
// finished tile is turned round in LDS so that the epilogue (bias, residual, activation, bf16)
// reads the residual and writes the output in whole 16-byte groups of 8 channels.
//
// Layers with few output pixels and a deep K cannot fill 256 compute units with output tiles
// alone; their K range is split over gridDim.y workgroups that store fp32 partial tiles into a
// workspace, and a second small kernel sums the slices and applies the epilogue.
#include "conv_common.h"


namespace ens {

constexpr int PRE_MAXK = 2048;   // most input channels a pre-activated 1x1 layer may have in the DMA kernel

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* global_ptr_t;

// LDS reads are issued as inline assembly so that the compiler does not serialise them against
// the asynchronous loads still in flight for later stages; the waits are placed by hand.
template <int OFFSET>
__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
    return v;
}

// Bytes of the ring of a tile shape: NS stages of (BP + BC) rows, or the first chunk of the staged output tile if larger.
template <int BP, int BC, int NS, int BKT>
constexpr int igemm_ring_bytes() {
    return NS * (BP + BC) * BKT * 2 > 32 * (BC + 4) * 4 ? NS * (BP + BC) * BKT * 2 : 32 * (BC + 4) * 4;
}

template <int BP, int BC, int WP, int WC, int NS, int BKT, bool PRE = false>
__global__ __launch_bounds__(256) void conv_igemm_bf16(const ConvArgs* __restrict__ argv, const int nb_) {
    ConvArgs a = argv[blockIdx.z];
    a.nb = nb_;
    const int P = nb_ * a.Ho * a.Wo, K = a.kh * a.kw * a.cin;
    static_assert(WP * WC == 4, "four wavefronts per workgroup");
    constexpr int WTP = BP / WP, WTC = BC / WC;      // wave tile
    constexpr int TP = WTP / 32, TC = WTC / 32;      // 32x32 blocks per wave
    static_assert(TP >= 1 && TC >= 1 && TP <= 4 && TC <= 4, "wave tile of 1..4 blocks per side");
    static_assert(BKT == 32 || BKT == 64, "K tile of 32 or 64 elements");
    constexpr int CH = BKT / 8;                      // 16-byte chunks per LDS row
    constexpr int RS = 256 / CH;                     // a thread serves rows r0 + RS*i
    constexpr int ROWB = BKT * 2;                    // bytes per LDS row
    static_assert(BP % RS == 0 && BC % RS == 0, "tiles are multiples of the row step");
    constexpr int NPL = BP / RS, NCL = BC / RS;      // asynchronous loads per thread and K tile
    constexpr int NLOAD = NPL + NCL;
    constexpr int STAGE = (BP + BC) * ROWB;          // bytes per ring stage
    static_assert(NS >= 2 && (NS - 2) * NLOAD <= 63, "outstanding loads must fit the wait counter");

    constexpr int OROW = BC + 4;                     // floats per pixel row of the staged output tile
    constexpr int RING = igemm_ring_bytes<BP, BC, NS, BKT>();
    // the output tile is staged through the ring in chunks of HROWS pixel rows
    constexpr int HFIT = RING / (OROW * 4) / 32 * 32;
    constexpr int HROWS = HFIT >= BP ? BP : (HFIT >= BP / 2 ? BP / 2 : (HFIT >= BP / 4 ? BP / 4 : 32));
    static_assert(HROWS >= 32 && BP % HROWS == 0 && HROWS * OROW * 4 <= RING, "output staging chunk");
    extern __shared__ __attribute__((aligned(1024))) unsigned char ring[];   // RING bytes, given at the launch
    // PRE (1x1 layers with a pre-activation): relu(x * scale + shift) per input channel is applied to
    // the pixel fragments on their way from LDS to the matrix cores; scale and shift of all K
    // channels wait in LDS (zero past K, so the zero-filled K tail stays zero).
    __shared__ __attribute__((aligned(16))) float pre_s[PRE ? PRE_MAXK + 64 : 4], pre_h[PRE ? PRE_MAXK + 64 : 4];

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);     // wave-uniform: LDS stage bases stay scalar
    const int wp0 = (wave % WP) * WTP, wc0 = (wave / WP) * WTC;
    const int n_ptiles = (P + BP - 1) / BP, n_ctiles = (a.cout + BC - 1) / BC;
    int ptile, ctile;
    tile_of_block(n_ptiles, n_ctiles, &ptile, &ctile);
    // a launch may carry argument blocks of a convolution with more output channels than this one
    // (two operations in one launch): the workgroups past this block's own tiles have nothing to do
    if (ptile >= n_ptiles) return;
    const int p0 = ptile * BP, c0 = ctile * BC;

    if constexpr (PRE) {
        for (int k = threadIdx.x; k < PRE_MAXK + 64; k += 256) {
            pre_s[k] = k < K ? a.pre_scale[k] : 0.f;
            pre_h[k] = k < K ? a.pre_shift[k] : 0.f;
        }
        __syncthreads();
    }
    // ---- this workgroup's share of the K tiles
    const int nk_all = (K + BKT - 1) / BKT;
    const int per_split = (nk_all + gridDim.y - 1) / gridDim.y;
    const int kt0 = blockIdx.y * per_split;
    const int nk = max(0, min(nk_all, kt0 + per_split) - kt0);

    // ---- load side: this thread fills slot (t % CH) of rows r0 + RS*i with chunk cchunk; the
    //      swizzle key is (r >> 1) & 7 for 128-byte rows and (r >> 2) & 3 for 64-byte rows.
    // Loads go through buffer descriptors: a lane whose byte offset lies past the end of the
    // buffer gets zeros written to its LDS slot, which is how padding taps, rows past the last
    // pixel, channels past the last output channel and the K tail are filled.
    constexpr unsigned OOB = 0xFFFFFFF0u;
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.x.p, 0, (int)((unsigned)nb_ * (unsigned)(a.H * a.W) * (unsigned)a.x.stride * 2u), 0x00020000);
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.w, 0, (int)((unsigned)a.cout * (unsigned)K * 2u), 0x00020000);
    const int r0 = t / CH;
    const int cchunk = (t % CH) ^ (CH == 8 ? (r0 >> 1) & 7 : (r0 >> 2) & 3);
    const int cpt = a.cin >> 3;                                  // 16-byte chunks per filter tap
    const int ntaps = a.kh * a.kw;
    // Per pixel row: byte offset of the window origin and the taps that fall inside the image,
    // bit kh of the low half-word for filter rows, bit 16 + kw for filter columns.
    unsigned rowoff[NPL], tapmask[NPL];
#pragma unroll
    for (int i = 0; i < NPL; i++) {
        const int p = p0 + r0 + RS * i;
        rowoff[i] = 0;
        tapmask[i] = 0;                                          // rows past the end: no tap is valid
        if (p < P) {
            // p -> (image, row, column) with one double multiply per division and a correction step
            int n = (int)((double)p * a.inv_hw);
            int rem = p - n * (a.Ho * a.Wo);
            if (rem < 0) { n--; rem += a.Ho * a.Wo; } else if (rem >= a.Ho * a.Wo) { n++; rem -= a.Ho * a.Wo; }
            int ho = (int)((double)rem * a.inv_w);
            int wo = rem - ho * a.Wo;
            if (wo < 0) { ho--; wo += a.Wo; } else if (wo >= a.Wo) { ho++; wo -= a.Wo; }
            const int hi0 = ho * a.sh - a.pt, wi0 = wo * a.sw - a.pl;
            unsigned m = 0;
            for (int k = 0; k < a.kh; k++) m |= (unsigned)(hi0 + k) < (unsigned)a.H ? 1u << k : 0u;
            for (int k = 0; k < a.kw; k++) m |= (unsigned)(wi0 + k) < (unsigned)a.W ? 0x10000u << k : 0u;
            tapmask[i] = m;
            rowoff[i] = (unsigned)((((n * a.H + hi0) * a.W + wi0) * a.x.stride + a.x.c0) * 2);
        }
    }
    unsigned wrowoff[NCL];                                       // byte offset of the weight row
#pragma unroll
    for (int i = 0; i < NCL; i++) {
        const int r = r0 + RS * i;
        wrowoff[i] = c0 + r < a.cout ? (unsigned)(c0 + r) * (unsigned)K * 2u : OOB;
    }

    // Position of this thread's chunk in the K walk: chunk kc -> filter tap (khi, kwi) and channel
    // chunk cq inside the tap; tapbase is the tap's byte offset from the window origin.  The
    // start comes from a division (the quotients are at most a few dozen, so a float multiply with
    // a half-step guard is exact); after that every K tile moves CH chunks on with adds and
    // selects when a tap holds at least CH chunks, and by division otherwise (narrow inputs).
    int kc = kt0 * CH + cchunk;
    const float inv_cpt = 1.0f / (float)cpt, inv_kw = 1.0f / (float)a.kw;
    int tap, cq, khi, kwi, tapbase;
    auto locate = [&]() {
        tap = (int)(((float)kc + 0.5f) * inv_cpt);
        cq = kc - tap * cpt;
        khi = (int)(((float)tap + 0.5f) * inv_kw);
        kwi = tap - khi * a.kw;
        tapbase = (khi * a.W + kwi) * a.x.stride * 2;
    };
    locate();
    const bool wide = cpt >= CH;
    const int col_step = a.x.stride * 2;                         // one tap to the right
    const int row_step = (a.W - a.kw) * a.x.stride * 2;          // from past the last tap of a filter row to the next row
    int issued = 0;                                              // K tiles issued so far

    // Issues the NLOAD asynchronous loads of the next K tile into ring stage `stage`.  Tiles past
    // the end of this workgroup's range are all zeros: the number of loads per iteration stays
    // constant, which the wait counter arithmetic below relies on.
    auto issue_tile = [&](int stage) {
        const bool in_range = issued < nk;
        const bool live = in_range && tap < ntaps;
        const unsigned need = live ? (1u << khi) | (0x10000u << kwi) : 0xFFFFFFFFu;   // both bits, or never
        const unsigned off = (unsigned)(tapbase + cq * 16);
        unsigned char* base = ring + stage * STAGE + wave * 1024;
#pragma unroll
        for (int i = 0; i < NPL; i++) {
            const unsigned o = (tapmask[i] & need) == need ? rowoff[i] + off : OOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (lds_ptr_t)(base + i * 4096), LDS_LOAD_BYTES, o, 0, 0, 0);
        }
        const bool k_ok = in_range && kc * 8 < K;
        const unsigned koffs = (unsigned)kc * 16u;
#pragma unroll
        for (int i = 0; i < NCL; i++) {
            const unsigned o = k_ok && wrowoff[i] != OOB ? wrowoff[i] + koffs : OOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wres, (lds_ptr_t)(base + (NPL + i) * 4096), LDS_LOAD_BYTES, o, 0, 0, 0);
        }
        // on to the next K tile
        issued++;
        kc += CH;
        if (wide) {
            cq += CH;
            const bool wrap = cq >= cpt;
            cq -= wrap ? cpt : 0;
            tap += wrap ? 1 : 0;
            kwi += wrap ? 1 : 0;
            tapbase += wrap ? col_step : 0;
            const bool wrap2 = kwi == a.kw;
            kwi = wrap2 ? 0 : kwi;
            khi += wrap2 ? 1 : 0;
            tapbase += wrap2 ? row_step : 0;
        } else {
            locate();
        }
    };

    f32x16 acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int j = 0; j < TP; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

    // ---- fragment side: lane reads row (lane & 31) of each 32-row block, chunk 2*ks + lane/32
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int lsw = CH == 8 ? (lrow >> 1) & 7 : (lrow >> 2) & 3;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)ring;
    const uint32_t xrow_addr = lds0 + (uint32_t)(wp0 + lrow) * ROWB;
    const uint32_t wrow_addr = lds0 + (uint32_t)(BP + wc0 + lrow) * ROWB;
    constexpr int BLK = 32 * ROWB;                               // bytes between 32-row blocks
    uint32_t koff[BKT / 16];
#pragma unroll
    for (int ks = 0; ks < BKT / 16; ks++) koff[ks] = (uint32_t)(((ks * 2 + lhalf) ^ lsw) * 16);

#pragma unroll
    for (int s = 0; s < NS - 1; s++) issue_tile(s);

    int stage = 0;
    for (int kt = 0; kt < nk; kt++) {
        // tile kt has landed once at most (NS-2) younger tiles of this wave are still in flight;
        // the barrier extends that to every wave's loads and also says that everybody is done
        // reading the stage that is refilled next
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * NLOAD) : "memory");
        __builtin_amdgcn_s_barrier();
        {
            int nxt = stage + NS - 1;
            if (nxt >= NS) nxt -= NS;
            issue_tile(nxt);
        }
        const uint32_t xs = xrow_addr + (uint32_t)stage * STAGE, ws = wrow_addr + (uint32_t)stage * STAGE;
        bf16x8 wf[2][TC], xf[2][TP];
        f32x4 ps[2][2], ph[2][2];                                // PRE: scale / shift of the step's 8 channels
        auto read_frags = [&](int ks, int b) {
            if constexpr (PRE) {
                const int kb = (kt0 + kt) * BKT + (ks * 2 + lhalf) * 8;
                ps[b][0] = *(const f32x4*)&pre_s[kb]; ps[b][1] = *(const f32x4*)&pre_s[kb + 4];
                ph[b][0] = *(const f32x4*)&pre_h[kb]; ph[b][1] = *(const f32x4*)&pre_h[kb + 4];
            }
            const uint32_t xa = xs + koff[ks], wa = ws + koff[ks];
            wf[b][0] = lds_read_b128<0>(wa);
            if (TC > 1) wf[b][1 % TC] = lds_read_b128<BLK>(wa);
            if (TC > 2) wf[b][2 % TC] = lds_read_b128<2 * BLK>(wa);
            if (TC > 3) wf[b][3 % TC] = lds_read_b128<3 * BLK>(wa);
            xf[b][0] = lds_read_b128<0>(xa);
            if (TP > 1) xf[b][1 % TP] = lds_read_b128<BLK>(xa);
            if (TP > 2) xf[b][2 % TP] = lds_read_b128<2 * BLK>(xa);
            if (TP > 3) xf[b][3 % TP] = lds_read_b128<3 * BLK>(xa);
        };
        read_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < BKT / 16; ks++) {
            const int b = ks & 1;
            // the fragments of this step are complete; tie them to the wait so that no matrix-core
            // instruction is scheduled ahead of it
            if constexpr (TC == 1 && TP == 1) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wf[b][0]), "+v"(xf[b][0]));
            else if constexpr (TC == 1 && TP == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wf[b][0]), "+v"(xf[b][0]), "+v"(xf[b][1]));
            else if constexpr (TC == 2 && TP == 1) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wf[b][0]), "+v"(wf[b][1]), "+v"(xf[b][0]));
            else if constexpr (TC == 2 && TP == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wf[b][0]), "+v"(wf[b][1]), "+v"(xf[b][0]), "+v"(xf[b][1]));
            else if constexpr (TC == 1 && TP == 4) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wf[b][0]), "+v"(xf[b][0]), "+v"(xf[b][1]), "+v"(xf[b][2]), "+v"(xf[b][3]));
            else if constexpr (TC == 2 && TP == 4) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wf[b][0]), "+v"(wf[b][1]), "+v"(xf[b][0]), "+v"(xf[b][1]), "+v"(xf[b][2]), "+v"(xf[b][3]));
            else if constexpr (TC == 4 && TP == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wf[b][0]), "+v"(wf[b][1]), "+v"(wf[b][2]), "+v"(wf[b][3]), "+v"(xf[b][0]), "+v"(xf[b][1]));
            else static_assert(TC * TP == 0, "unsupported wave tile");
            if (ks + 1 < BKT / 16) read_frags(ks + 1, b ^ 1);     // next step's reads fly under this step's MFMAs
            if constexpr (PRE) {
#pragma unroll
                for (int j = 0; j < TP; j++) {
                    u32x4 u = __builtin_bit_cast(u32x4, xf[b][j]);
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const float lo = __uint_as_float(u[q] << 16), hi = __uint_as_float(u[q] & 0xFFFF0000u);
                        const float sl = ps[b][q >> 1][(2 * q) & 3], sh = ps[b][q >> 1][(2 * q + 1) & 3];
                        const float hl = ph[b][q >> 1][(2 * q) & 3], hh = ph[b][q >> 1][(2 * q + 1) & 3];
                        u[q] = pack_bf16x2(fmaxf(fmaf(lo, sl, hl), 0.f), fmaxf(fmaf(hi, sh, hh), 0.f));
                    }
                    xf[b][j] = __builtin_bit_cast(bf16x8, u);
                }
            }
#pragma unroll
            for (int i = 0; i < TC; i++)
#pragma unroll
                for (int j = 0; j < TP; j++)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[b][i], xf[b][j], acc[i][j], 0, 0, 0);
        }
        if (++stage == NS) stage = 0;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");             // drain the trailing (all-zero) loads
    __syncthreads();                                             // everybody is done with the ring

    // ---- epilogue.  An accumulator lane holds one pixel (lane & 31) and, in register v, channel
    // 8*(v/4) + 4*(lane/32) + v%4 of its 32x32 block: runs of four channels at a stride of one
    // pixel, which would reach memory as scattered 8-byte pieces.  The tile is therefore turned
    // round in LDS (fp32, rows padded by 16 bytes against bank conflicts) and leaves the workgroup
    // as whole 16-byte groups of 8 channels, a pixel's channels side by side in one line.
    float* otile = (float*)ring;
    constexpr int G = BC / 8;                                    // 8-channel groups per pixel row
    const bool split = gridDim.y > 1;
    float* mine = split ? a.ws + (size_t)blockIdx.y * P * a.cout : nullptr;
    uint16_t* __restrict__ yg = (uint16_t*)a.y.p;
    const uint16_t* __restrict__ rg = (const uint16_t*)a.res.p;
#pragma unroll
    for (int h0 = 0; h0 < BP; h0 += HROWS) {
        if (h0 > 0) __syncthreads();                             // previous chunk has left LDS
#pragma unroll
        for (int j = 0; j < TP; j++) {
            const int rb = wp0 + j * 32;                         // first pixel row of this block
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
        for (int it = 0; it < HROWS * G / 256; it++) {
            const int e = t + 256 * it;
            const int row = e / G, g = e - row * G;
            const int p = p0 + h0 + row, co = c0 + g * 8;
            if (p >= P || co >= a.cout) continue;
            const float4 lo = *(const float4*)&otile[row * OROW + g * 8];
            const float4 hi = *(const float4*)&otile[row * OROW + g * 8 + 4];
            if (split) {                                         // fp32 partial sums of this K split
                float* d = mine + (size_t)p * a.cout + co;
                *ENS_GLOBAL_W(f32x4, d) = f32x4{lo.x, lo.y, lo.z, lo.w};
                *ENS_GLOBAL_W(f32x4, d + 4) = f32x4{hi.x, hi.y, hi.z, hi.w};
                continue;
            }
            const f32x4 b0 = *ENS_GLOBAL(f32x4, a.bias + co), b1 = *ENS_GLOBAL(f32x4, a.bias + co + 4);
            const f32x4 s0 = *ENS_GLOBAL(f32x4, a.scale + co), s1 = *ENS_GLOBAL(f32x4, a.scale + co + 4);
            float v[8] = {fmaf(lo.x, s0.x, b0.x), fmaf(lo.y, s0.y, b0.y), fmaf(lo.z, s0.z, b0.z), fmaf(lo.w, s0.w, b0.w),
                          fmaf(hi.x, s1.x, b1.x), fmaf(hi.y, s1.y, b1.y), fmaf(hi.z, s1.z, b1.z), fmaf(hi.w, s1.w, b1.w)};
            if (rg) {
                const u32x4 r = *ENS_GLOBAL(u32x4, rg + (size_t)p * a.res.stride + a.res.c0 + co);
                const uint32_t rr[4] = {r.x, r.y, r.z, r.w};
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
            *ENS_GLOBAL_W(u32x4, yg + (size_t)p * a.y.stride + a.y.c0 + co) = u32x4{o[0], o[1], o[2], o[3]};
        }
    }
}

// Second pass of a split convolution: sums the fp32 slices and applies bias, residual and
// activation; one thread per pixel and run of four output channels.
__global__ void conv_splitk_epilogue(const ConvArgs* __restrict__ argv, const int nb_, const int splits) {
    const ConvArgs a = argv[blockIdx.z];
    const int P = nb_ * a.Ho * a.Wo;
    const int cq = a.cout >> 2;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long long)P * cq) return;
    const int co = (int)(idx % cq) * 4;
    const long long p = idx / cq;
    const size_t slice = (size_t)P * a.cout;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int sp = 0; sp < splits; sp++) {
        const float4 v = *(const float4*)(a.ws + sp * slice + (size_t)p * a.cout + co);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    const float4 b = *(const float4*)(a.bias + co), m = *(const float4*)(a.scale + co);
    float v[4] = {fmaf(s.x, m.x, b.x), fmaf(s.y, m.y, b.y), fmaf(s.z, m.z, b.z), fmaf(s.w, m.w, b.w)};
    if (a.res.p) {
        const uint2 r = *(const uint2*)((const uint16_t*)a.res.p + (size_t)p * a.res.stride + a.res.c0 + co);
        v[0] += bf16_to_f32((uint16_t)(r.x & 0xFFFF));
        v[1] += bf16_to_f32((uint16_t)(r.x >> 16));
        v[2] += bf16_to_f32((uint16_t)(r.y & 0xFFFF));
        v[3] += bf16_to_f32((uint16_t)(r.y >> 16));
    }
    apply_act_n<4>(v, a.act);
    uint2 o;
    o.x = pack_bf16x2(v[0], v[1]);
    o.y = pack_bf16x2(v[2], v[3]);
    *(uint2*)((uint16_t*)a.y.p + (size_t)p * a.y.stride + a.y.c0 + co) = o;
}

hipError_t launch_conv_splitk_epilogue(const ConvArgs& a, const ConvArgs* argv, int G, int nb, int P, int splits, hipStream_t s) {
    const long long work = (long long)P * (a.cout / 4);
    ENS_LAUNCH_LAST(conv_splitk_epilogue, dim3((unsigned)((work + 255) / 256), 1, G), dim3(256), 0, s, argv, nb, splits);
    return hipGetLastError();
}

double conv_flops(const ConvArgs& a, int nb) {
    return 2.0 * (double)nb * a.Ho * a.Wo * a.cout * a.kh * a.kw * a.cin;
}

// ---- tile and split choice ---------------------------------------------------------------
// Measured on MI355X over the layer shapes of residual, dense and inception networks at batch
// 8-128: what counts most is how many workgroups a compute unit holds at once (their load,
// matrix-core and store phases overlap), so the tiles are small and the ring is two stages deep:
// 32 KB of LDS per workgroup, five workgroups per compute unit.
struct Variant { int bp, bc, bk; const char* name; };
static const Variant VARIANTS[] = {
    {128, 32, 64, "conv_igemm_bf16<128,32,k64>"},    // narrow outputs (dense-block growth layers)
    {64, 64, 64, "conv_igemm_bf16<64,64,k64>"},      // small grids
    {64, 64, 32, "conv_igemm_bf16<64,64,k32>"},      // small grids, shallow K
    {128, 64, 64, "conv_igemm_bf16<128,64,k64>"},    // grids that fill the chip, deep K
    {128, 64, 32, "conv_igemm_bf16<128,64,k32>"},    // grids that fill the chip, shallow K
    {128, 128, 64, "conv_igemm_bf16<128,128,k64>"},  // many pixels, wide outputs, deep K: a third less load traffic per flop
};

// A gang of G members multiplies the grid by G.  When 128x64 tiles still give two workgroups per
// compute unit they are taken (a third less L2-to-LDS traffic per flop than 64x64); otherwise
// the 64x64 tile keeps more workgroups in flight.
static int pick_variant(const ConvArgs& a, long long P, long long K, int G) {
    if (a.cout <= 32) return 0;
    const long long t12864 = G * ((P + 127) / 128) * ((a.cout + 63) / 64);
    const long long t128128 = G * ((P + 127) / 128) * ((a.cout + 127) / 128);
    if (a.cout % 128 == 0 && K > 640 && t128128 >= 3 * cu_budget()) return 5;   // no channel tile half empty
    if (t12864 >= 2 * cu_budget()) return K <= 640 ? 4 : 3;
    return K <= 256 ? 2 : 1;
}

// Splits of the K range for launches that would leave compute units idle.  Each split keeps at
// least four K tiles; the workspace holds one P * cout slice of floats per split.
static int pick_splits(const ConvArgs& a, long long P, long long K, int variant, int G) {
    if (!a.ws) return 1;
    const Variant& v = VARIANTS[variant];
    const long long tiles = G * ((P + v.bp - 1) / v.bp) * ((a.cout + v.bc - 1) / v.bc);
    const long long nk = (K + v.bk - 1) / v.bk;
    if (tiles >= 2 * cu_budget() || nk < 8) return 1;
    long long s = (3 * cu_budget() + tiles - 1) / tiles;
    s = s < nk / 4 ? s : nk / 4;
    if (s > 16) s = 16;
    while (s > 1 && s * P * a.cout > a.ws_floats) s--;
    return s < 1 ? 1 : (int)s;
}

// Pre-activated layers the DMA kernel takes: 1x1, stride 1, no padding (k = input channel), K within
// the LDS table.  Others go to the register-staged kernel.
static bool pre_in_dma_kernel(const ConvArgs& a) {
    bool ok = a.kh == 1 && a.kw == 1 && a.sh == 1 && a.sw == 1 && a.pt == 0 && a.pl == 0 && a.cin <= PRE_MAXK;
    return ok;
}

const char* conv_bf16_variant_name(const ConvArgs& a, int G) {
    const long long P = (long long)a.nb * a.Ho * a.Wo;
    if (a.pre_scale && !pre_in_dma_kernel(a)) return conv_regstage_name(a, (int)P);
    if (conv_pw_applicable(a, a.nb, G)) return conv_pw_name(a, G);
    if (conv_taps_applicable(a, a.nb)) return conv_taps_name(a);
    if (conv_wreg_applicable(a, a.nb, G)) return conv_wreg_name(a);
    if (const int hv = conv_halo_pick(a, a.nb, G); hv >= 0) return conv_halo_name(hv);
    return VARIANTS[pick_variant(a, P, (long long)a.kh * a.kw * a.cin, G)].name;
}

template <int BP, int BC, int WP, int WC, int NS, int BKT = 64>
static hipError_t launch_variant(const ConvArgs& a, const ConvArgs* argv, int G, int nb, int P, int splits, hipStream_t s) {
    const dim3 grid(((P + BP - 1) / BP) * ((a.cout + BC - 1) / BC), splits, G);
    constexpr int ring = igemm_ring_bytes<BP, BC, NS, BKT>();
    // LDS above 64 KB (the ring plus the kernel's own tables) has to be asked for once per kernel
    auto raise = [&](const void* kernel, bool& raised) -> hipError_t {
        if (raised) return hipSuccess;
        hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, ring);
        raised = e == hipSuccess;
        return e;
    };
    if (a.pre_scale) {                                           // pre-activated 1x1: no K split (the launcher asks for none)
        if constexpr (ring + 2 * (PRE_MAXK + 64) * 4 > 64 * 1024) {
            static bool raised = false;
            if (hipError_t e = raise((const void*)&conv_igemm_bf16<BP, BC, WP, WC, NS, BKT, true>, raised); e != hipSuccess) return e;
        }
        ENS_LAUNCH((conv_igemm_bf16<BP, BC, WP, WC, NS, BKT, true>), grid, dim3(256), ring, s, argv, nb);
        return hipGetLastError();
    }
    if constexpr (ring + 64 > 64 * 1024) {
        static bool raised = false;
        if (hipError_t e = raise((const void*)&conv_igemm_bf16<BP, BC, WP, WC, NS, BKT>, raised); e != hipSuccess) return e;
    }
    if (splits > 1) ENS_LAUNCH_FIRST((conv_igemm_bf16<BP, BC, WP, WC, NS, BKT>), grid, dim3(256), ring, s, argv, nb);
    else ENS_LAUNCH((conv_igemm_bf16<BP, BC, WP, WC, NS, BKT>), grid, dim3(256), ring, s, argv, nb);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && splits > 1) e = launch_conv_splitk_epilogue(a, argv, G, nb, P, splits, s);
    return e;
}

hipError_t launch_conv_bf16(const ConvArgs& a, const ConvArgs* argv, int G, int nb, hipStream_t s) {
    // shapes the kernels assume: 16-byte groups of 8 channels on the way in and on the way out
    if (a.cin % 8 || a.x.stride % 8 || a.x.c0 % 8) return hipErrorInvalidValue;
    if (a.cout % 8 || a.y.stride % 8 || a.y.c0 % 8) return hipErrorInvalidValue;
    if (a.res.p && (a.res.stride % 8 || a.res.c0 % 8)) return hipErrorInvalidValue;
    if (nb <= 0 || a.cin <= 0 || a.cout <= 0 || !a.bias || !a.scale || G <= 0 || !argv) return hipErrorInvalidValue;
    if ((a.pre_scale == nullptr) != (a.pre_shift == nullptr)) return hipErrorInvalidValue;
    const long long P64 = (long long)nb * a.Ho * a.Wo;
    const long long K64 = (long long)a.kh * a.kw * a.cin;
    if (P64 <= 0 || P64 >= (1LL << 31) || K64 >= (1LL << 31)) return hipErrorInvalidValue;
    const int P = (int)P64;
    if (a.gate && (a.pre_scale || !conv_pw_applicable(a, nb, G))) return hipErrorInvalidValue;   // only the 1x1 kernel applies a gate
    if (a.pre_scale && !pre_in_dma_kernel(a)) return launch_conv_regstage(a, argv, G, nb, P, s);
    if (conv_pw_applicable(a, nb, G)) return launch_conv_pw(a, argv, G, nb, s);
    if (conv_taps_applicable(a, nb)) return launch_conv_taps(a, argv, G, nb, s);
    if (conv_wreg_applicable(a, nb, G)) return launch_conv_wreg(a, argv, G, nb, s);
    if (const int hv = conv_halo_pick(a, nb, G); hv >= 0) return launch_conv_halo(a, argv, G, nb, hv, s);
    // byte offsets inside the kernel are unsigned 32-bit, 0xFFFFFFF0 stands for 'out of range'
    if ((long long)nb * a.H * a.W * a.x.stride >= 0x7FFFFF00LL || (long long)a.cout * K64 >= 0x70000000LL || a.kh > 16 || a.kw > 16) return hipErrorInvalidValue;
    int variant = pick_variant(a, P64, K64, G);
    int splits = a.pre_scale ? 1 : pick_splits(a, P64, K64, variant, G);
    switch (variant) {
        case 0: return launch_variant<128, 32, 4, 1, 2, 64>(a, argv, G, nb, P, splits, s);
        case 2: return launch_variant<64, 64, 2, 2, 2, 32>(a, argv, G, nb, P, splits, s);
        case 3: return launch_variant<128, 64, 2, 2, 2, 64>(a, argv, G, nb, P, splits, s);
        case 4: return launch_variant<128, 64, 2, 2, 2, 32>(a, argv, G, nb, P, splits, s);
        case 5: return a.pre_scale ? launch_variant<128, 64, 2, 2, 2, 64>(a, argv, G, nb, P, splits, s)
                                   : launch_variant<128, 128, 2, 2, 2, 64>(a, argv, G, nb, P, splits, s);
        default: return launch_variant<64, 64, 2, 2, 2, 64>(a, argv, G, nb, P, splits, s);
    }
}

}  // namespace ens
