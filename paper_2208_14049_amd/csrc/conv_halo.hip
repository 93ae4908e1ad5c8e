// Stride-1 convolutions with "same" padding and a KH x KW filter (3x3, and the 1x7 / 7x1 / 1x3 / 3x1 filters of
// factorised inception modules) on the CDNA4 matrix cores with the input window held in LDS: every input
// pixel a workgroup needs is fetched once per channel block and serves all KH * KW filter taps, where the
// generic implicit-GEMM kernel fetches it once per tap.
//
// Pixels are numbered in a padded raster: with gh = (KH - 1) / 2 and gw = (KW - 1) / 2, image n, row hi,
// column wi sits at position
//   pp = (n * (H + gh) + hi) * (W + gw) + wi
// with gw extra columns per row and gh extra rows per image that hold no pixel.  In that raster
// the tap (dh, dw) of ANY output position is the position dh * (W + gw) + dw further on, and the
// neighbours that fall outside an image land on the extra columns / rows (to the left of a row on those of
// the row before, above an image on those of the image before): they are loaded as zeros
// (a buffer load past the end of its buffer writes zeros), so the filter taps need no masks and
// the fragment addresses of a tap differ from the centre's by one constant.  The price is
// matrix-core work on the padding positions themselves, (H+gh)(W+gw)/(HW) - 1 of the total.
//
// A workgroup of 4 wavefronts owns BP consecutive padded positions x BC output channels.  Its
// "halo" is the run of BP + (KH-1)(W+gw) + KW-1 positions those outputs read, CB channels wide, one LDS
// row of 2*CB bytes per position with the 16-byte chunks swizzled as in the generic kernel.  The
// loop runs over channel blocks and, inside, the taps; each step takes a BC x CB tile of
// the weights through a two-stage ring.  While block cb is being used the halo of block cb+1
// arrives in the second halo buffer, a slice of it with every tap.  All loads are asynchronous
// global-to-LDS loads; the weight loads' per-thread offsets are loop invariant (the moving part
// is the scalar offset), so the loop body is address-free apart from the fragment reads.
#include "conv_common.h"


namespace ens {

typedef __attribute__((address_space(3))) void* lds_ptr_t;

template <int OFFSET>
__device__ __forceinline__ bf16x8 halo_lds_read(uint32_t addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
    return v;
}

template <int KH, int KW, int BP, int BC, int WP, int WC, int CB, int NHL>
__global__ __launch_bounds__(256) void conv_halo_bf16(const ConvArgs* __restrict__ argv, const int nb_,
                                                      const int hrows, const int nbuf) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const ConvArgs a = argv[blockIdx.z];
    static_assert(WP * WC == 4, "four wavefronts per workgroup");
    constexpr int WTP = BP / WP, WTC = BC / WC;
    constexpr int TP = WTP / 32, TC = WTC / 32;
    static_assert(TP >= 1 && TC >= 1 && TP <= 2 && TC <= 2, "wave tile of 1..2 blocks per side");
    static_assert(CB == 32 || CB == 64, "channel block of 32 or 64");
    constexpr int CH = CB / 8;                       // 16-byte chunks per LDS row
    constexpr int RS = 256 / CH;                     // rows one load instruction of the workgroup covers
    constexpr int ROWB = CB * 2;
    static_assert(BC % RS == 0, "weight tile is a multiple of the row step");
    constexpr int NCL = BC / RS;                     // weight loads per thread and step
    constexpr int WSTAGE = BC * ROWB;                // bytes per stage of the weight ring
    constexpr int KS = CB / 16;                      // matrix-core steps per tap
    constexpr int NR = TC + TP;                      // LDS reads per matrix-core step

    constexpr int OROW = BC + 4;
    constexpr int MINLDS = 2 * WSTAGE + (BP + 32) * ROWB;        // ring + smallest possible halo
    constexpr int HFIT = MINLDS / (OROW * 4) / 32 * 32;
    constexpr int HROWS = HFIT >= BP ? BP : (HFIT >= BP / 2 ? BP / 2 : (HFIT >= BP / 4 ? BP / 4 : 32));
    static_assert(HROWS >= 32 && BP % HROWS == 0 && HROWS * OROW * 4 <= MINLDS, "output staging chunk");

    constexpr int NT = KH * KW, GH = (KH - 1) / 2, GW = (KW - 1) / 2;   // taps; gap rows per image and gap columns per row
    const int W1 = a.W + GW, H1 = a.H + GH, img = H1 * W1;
    const int origin = GH * W1 + GW;                 // from a tile's first halo row to its first output
    const int PP = nb_ * img;                        // padded positions of the batch
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wp0 = (wave % WP) * WTP, wc0 = (wave / WP) * WTC;
    const int n_ptiles = (PP + BP - 1) / BP, n_ctiles = (a.cout + BC - 1) / BC;
    int ptile, ctile;
    tile_of_block(n_ptiles, n_ctiles, &ptile, &ctile);
    const int pp0 = ptile * BP, c0 = ctile * BC;
    // gridDim.y workgroups share the channel blocks of one output tile; each stores fp32 partial
    // sums into its slice of the workspace and a second kernel adds the slices up
    const int ncb_all = a.cin / CB;
    const int per_split = (ncb_all + gridDim.y - 1) / gridDim.y;
    const int cb_begin = blockIdx.y * per_split;
    const int ncb = min(ncb_all, cb_begin + per_split);        // one past this workgroup's last block
    const int nsl = hrows / RS;                      // load instructions per halo block

    unsigned char* const halo = lds + 2 * WSTAGE;
    const int hbytes = hrows * ROWB;
    int* const tbl = (int*)(halo + nbuf * hbytes);   // halo row -> pixel index (n*H + hi)*W + wi, -1: padding

    // ---- which pixel each halo row is; row 0 is the top-left tap of the tile's first output
    raster_table(tbl, hrows, pp0 - origin, PP, H1, W1, a.H, a.W);
    __syncthreads();

    // ---- load side.  Offsets past the end of a buffer give zeros in LDS; 2^31 is past the end of
    //      every buffer the launcher admits and stays so when the scalar offset is added.
    constexpr unsigned OOBV = 0x80000000u;
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.x.p, 0, (int)((unsigned)nb_ * (unsigned)(a.H * a.W) * (unsigned)a.x.stride * 2u), 0x00020000);
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)a.w, 0, (int)((unsigned)a.cout * (unsigned)(NT * a.cin) * 2u), 0x00020000);
    const int r0 = t / CH;
    const int cchunk = (t % CH) ^ (CH == 8 ? (r0 >> 1) & 7 : (r0 >> 2) & 3);
    const unsigned xlane = (unsigned)(a.x.c0 * 2 + cchunk * 16);
    // slot s of a halo block: row r0 + RS*s, this thread's chunk.  Padding rows read 'outside'.
    auto issue_halo = [&](int buf, int s, int cb) {
        const int p = tbl[s * RS + r0];
        const unsigned vo = p >= 0 ? (unsigned)(p * a.x.stride * 2) + xlane : OOBV;
        unsigned char* base = halo + buf * hbytes + s * 4096 + wave * 1024;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (lds_ptr_t)base, LDS_LOAD_BYTES, vo, cb * CB * 2, 0, 0);
    };
    unsigned wvo[NCL];                               // weight row c0 + r0 + RS*i, this thread's chunk
#pragma unroll
    for (int i = 0; i < NCL; i++) {
        const int r = c0 + r0 + RS * i;
        wvo[i] = r < a.cout ? (unsigned)r * (unsigned)(NT * a.cin) * 2u + (unsigned)cchunk * 16u : OOBV;
    }
    auto issue_weights = [&](int stage, int cb, int tap) {
        const int so = (tap * a.cin + cb * CB) * 2;
        unsigned char* base = lds + stage * WSTAGE + wave * 1024;
#pragma unroll
        for (int i = 0; i < NCL; i++)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wres, (lds_ptr_t)(base + i * 4096), LDS_LOAD_BYTES, wvo[i], so, 0, 0);
    };

    // the first block's halo, four table look-ups at a time
    for (int s0 = 0; s0 < nsl; s0 += 4) {
        int p4[4];
#pragma unroll
        for (int j = 0; j < 4; j++) p4[j] = tbl[(s0 + j < nsl ? s0 + j : nsl - 1) * RS + r0];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            if (s0 + j >= nsl) break;
            const unsigned vo = p4[j] >= 0 ? (unsigned)(p4[j] * a.x.stride * 2) + xlane : OOBV;
            unsigned char* base = halo + (s0 + j) * 4096 + wave * 1024;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (lds_ptr_t)base, LDS_LOAD_BYTES, vo, cb_begin * CB * 2, 0, 0);
        }
    }
    issue_weights(0, cb_begin, 0);

    // ---- what the epilogue needs from memory is asked for now and is there long before it is used
    const bool split = gridDim.y > 1;
    const int* own = tbl + origin;                               // the centre tap's halo rows: this tile's outputs
    TilePrefetch<BP, BC> pf;
    pf.load(a, own, c0, split);

    f32x16 acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; i++)
#pragma unroll
        for (int j = 0; j < TP; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

    // ---- fragment side
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int lsw = CH == 8 ? (lrow >> 1) & 7 : (lrow >> 2) & 3;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
    const uint32_t wrow_addr = lds0 + (uint32_t)(wc0 + lrow) * ROWB;
    constexpr int BLK = 32 * ROWB;
    uint32_t koff[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) koff[ks] = (uint32_t)(((ks * 2 + lhalf) ^ lsw) * 16);
    const uint32_t halo0 = lds0 + 2 * WSTAGE;
    const uint32_t lq = (uint32_t)(wp0 + lrow);

    int stage = 0;
    // With one halo buffer (nbuf == 1) a block's halo is loaded when the previous block is done
    // with: the load is exposed once per block and the LDS saved lets more workgroups share the
    // compute unit; with two buffers it arrives during the previous block's taps.
    const bool single = nbuf == 1;
    for (int cb = cb_begin; cb < ncb; cb++) {
        const int hb = single ? 0 : (cb - cb_begin) & 1;         // halo buffer of this block
        const uint32_t hbuf = halo0 + (uint32_t)(hb * hbytes);
        const bool more = cb + 1 < ncb;
#pragma unroll
        for (int tap = 0; tap < NT; tap++) {
            // this step's weights (and, at tap 0, the block's halo) have landed; the barrier extends
            // that to the other waves' loads and says that nobody still reads what is refilled next
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            if (tap == 0 && single && cb > cb_begin) {           // everybody is done with the previous block's halo
                for (int s = 0; s < nsl; s++) issue_halo(0, s, cb);
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
            }
            if (tap < NT - 1) issue_weights(stage ^ 1, cb, tap + 1);
            else if (more) issue_weights(stage ^ 1, cb + 1, 0);
            if (more && !single) {
#pragma unroll
                for (int j = 0; j < NHL; j++)
                    if (tap * NHL + j < nsl) issue_halo(hb ^ 1, tap * NHL + j, cb + 1);
            }
            // tap (dh, dw): dh rows of the padded raster down, dw positions to the right
            const uint32_t q = lq + (uint32_t)((tap / KW) * W1 + tap % KW);
            const uint32_t key = CH == 8 ? (q >> 1) & 7 : (q >> 2) & 3;
            const uint32_t xs = hbuf + q * ROWB + ((((uint32_t)lhalf) ^ key) << 4);
            const uint32_t ws = wrow_addr + (uint32_t)stage * WSTAGE;
            bf16x8 wf[2][TC], xf[2][TP];
            auto read_frags = [&](int ks, int b) {
                const uint32_t xa = xs ^ (uint32_t)(ks << 5), wa = ws + koff[ks];
                wf[b][0] = halo_lds_read<0>(wa);
                if (TC > 1) wf[b][1 % TC] = halo_lds_read<BLK>(wa);
                xf[b][0] = halo_lds_read<0>(xa);
                if (TP > 1) xf[b][1 % TP] = halo_lds_read<BLK>(xa);
            };
            read_frags(0, 0);
#pragma unroll
            for (int ks = 0; ks < KS; ks++) {
                const int b = ks & 1;
                // The next step's reads are issued first; LDS returns in order, so once no more than
                // those NR are outstanding this step's fragments are complete.  They are tied to
                // the wait so that no matrix-core instruction is scheduled ahead of it.
                if (ks + 1 < KS) read_frags(ks + 1, b ^ 1);
#define ENS_HALO_WAIT(N)                                                                                                   \
    if constexpr (TC == 1 && TP == 1) asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(wf[b][0]), "+v"(xf[b][0]) : "n"(N));       \
    else if constexpr (TC == 1 && TP == 2) asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(wf[b][0]), "+v"(xf[b][0]), "+v"(xf[b][1]) : "n"(N)); \
    else if constexpr (TC == 2 && TP == 1) asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(wf[b][0]), "+v"(wf[b][1]), "+v"(xf[b][0]) : "n"(N)); \
    else asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(wf[b][0]), "+v"(wf[b][1]), "+v"(xf[b][0]), "+v"(xf[b][1]) : "n"(N));
                if (ks + 1 < KS) { ENS_HALO_WAIT(NR) } else { ENS_HALO_WAIT(0) }
#undef ENS_HALO_WAIT
#pragma unroll
                for (int i = 0; i < TC; i++)
#pragma unroll
                    for (int j = 0; j < TP; j++)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[b][i], xf[b][j], acc[i][j], 0, 0, 0);
            }
            stage ^= 1;
        }
    }
    __syncthreads();                                             // everybody is done with ring and halo

    // ---- epilogue; positions of the padded raster that hold no pixel are dropped there
    store_tile<BP, BC, TP, TC, HROWS>(a, acc, (float*)lds, own, pf, wp0, wc0, split, blockIdx.y, nb_ * a.H * a.W);
}

// ---- host side -----------------------------------------------------------------------------
// name: the kernel instance (the one- and two-buffer forms of a tile are the same instance)
struct HaloVariant { int kh, kw, bp, bc, cb, nhl; bool single; const char* name; };
static const HaloVariant HALO_VARIANTS[] = {
    {3, 3, 128, 64, 64, 1, false, "conv3x3_halo_bf16<128,64,c64>"},
    {3, 3, 256, 64, 64, 2, false, "conv3x3_halo_bf16<256,64,c64>"},
    {3, 3, 128, 128, 64, 1, false, "conv3x3_halo_bf16<128,128,c64>"},
    {3, 3, 256, 64, 32, 1, false, "conv3x3_halo_bf16<256,64,c32>"},
    {3, 3, 128, 64, 32, 1, false, "conv3x3_halo_bf16<128,64,c32>"},
    {3, 3, 128, 128, 32, 1, false, "conv3x3_halo_bf16<128,128,c32>"},
    {3, 3, 128, 64, 64, 1, true, "conv3x3_halo_bf16<128,64,c64>"},
    {3, 3, 256, 64, 64, 2, true, "conv3x3_halo_bf16<256,64,c64>"},
    {3, 3, 128, 128, 64, 1, true, "conv3x3_halo_bf16<128,128,c64>"},
    {3, 3, 128, 64, 32, 1, true, "conv3x3_halo_bf16<128,64,c32>"},
    {3, 3, 256, 64, 32, 1, true, "conv3x3_halo_bf16<256,64,c32>"},
    {3, 3, 128, 128, 32, 1, true, "conv3x3_halo_bf16<128,128,c32>"},
    {3, 3, 256, 32, 64, 2, true, "conv3x3_halo_bf16<256,32,c64>"},
    {3, 3, 256, 32, 64, 2, false, "conv3x3_halo_bf16<256,32,c64>"},
    // the one-dimensional filters, four entries each from HALO_LINE on: 64-channel blocks with two halo buffers
    // and with one, 32-channel blocks with two and with one (the two forms are one kernel instance)
    {1, 7, 128, 64, 64, 1, false, "conv1x7_halo_bf16<128,64,c64>"},
    {1, 7, 128, 64, 64, 1, true, "conv1x7_halo_bf16<128,64,c64>"},
    {1, 7, 128, 64, 32, 1, false, "conv1x7_halo_bf16<128,64,c32>"},
    {1, 7, 128, 64, 32, 1, true, "conv1x7_halo_bf16<128,64,c32>"},
    {7, 1, 128, 64, 64, 2, false, "conv7x1_halo_bf16<128,64,c64>"},
    {7, 1, 128, 64, 64, 2, true, "conv7x1_halo_bf16<128,64,c64>"},
    {7, 1, 128, 64, 32, 1, false, "conv7x1_halo_bf16<128,64,c32>"},
    {7, 1, 128, 64, 32, 1, true, "conv7x1_halo_bf16<128,64,c32>"},
    {1, 3, 128, 64, 64, 2, false, "conv1x3_halo_bf16<128,64,c64>"},
    {1, 3, 128, 64, 64, 2, true, "conv1x3_halo_bf16<128,64,c64>"},
    {1, 3, 128, 64, 32, 1, false, "conv1x3_halo_bf16<128,64,c32>"},
    {1, 3, 128, 64, 32, 1, true, "conv1x3_halo_bf16<128,64,c32>"},
    {3, 1, 128, 64, 64, 2, false, "conv3x1_halo_bf16<128,64,c64>"},
    {3, 1, 128, 64, 64, 2, true, "conv3x1_halo_bf16<128,64,c64>"},
    {3, 1, 128, 64, 32, 1, false, "conv3x1_halo_bf16<128,64,c32>"},
    {3, 1, 128, 64, 32, 1, true, "conv3x1_halo_bf16<128,64,c32>"},
};
constexpr int HALO_LINE = 14;                        // first entry of the one-dimensional filters
constexpr int N_HALO_VARIANTS = sizeof(HALO_VARIANTS) / sizeof(HALO_VARIANTS[0]);
constexpr int LDS_LIMIT = 160 * 1024;


// Splits of the channel blocks for launches with fewer output tiles than compute units: as many
// as give about two workgroups per compute unit, each with at least two channel blocks, within
// the workspace (one P x cout fp32 slice per split).  With one tile per compute unit or more the
// extra pass over fp32 partial sums costs more than the idle units (measured).
static long long halo_positions(const ConvArgs& a, int nb) {   // of the padded raster
    return (long long)nb * (a.H + (a.kh - 1) / 2) * (a.W + (a.kw - 1) / 2);
}

static int halo_splits(const ConvArgs& a, const HaloVariant& v, int nb, int G) {
    if (!a.ws) return 1;
    const long long PP = halo_positions(a, nb), P = (long long)nb * a.H * a.W;
    const long long tiles = G * ((PP + v.bp - 1) / v.bp) * ((a.cout + v.bc - 1) / v.bc);
    const int ncb = a.cin / v.cb;
    if (tiles >= cu_budget() || ncb < 4) return 1;
    long long s = (2 * cu_budget() + tiles - 1) / tiles;
    s = s < ncb / 2 ? s : ncb / 2;
    if (s > 8) s = 8;
    while (s > 1 && s * P * a.cout > a.ws_floats) s--;
    if (s <= 1) return 1;
    const int per = (ncb + (int)s - 1) / (int)s;
    return (ncb + per - 1) / per;                                // no empty split
}

// Rows and bytes of LDS variant v needs for this layer; false when it does not fit.
static bool halo_layout(const ConvArgs& a, const HaloVariant& v, int splits, int* hrows, int* nbuf, size_t* bytes) {
    if (a.cin % v.cb || a.kh != v.kh || a.kw != v.kw) return false;
    const int rs = 256 / (v.cb / 8);
    const int need = v.bp + (a.kh - 1) * (a.W + (a.kw - 1) / 2) + a.kw - 1;
    const int rows = (need + rs - 1) / rs * rs;
    const int ncb = a.cin / v.cb, per = (ncb + splits - 1) / splits;
    *hrows = rows;
    *nbuf = per > 1 && !v.single ? 2 : 1;
    // the blocks after the first arrive nhl load slots per tap
    if (*nbuf == 2 && rows / rs > a.kh * a.kw * v.nhl) return false;
    *bytes = (size_t)2 * v.bc * v.cb * 2 + (size_t)*nbuf * rows * v.cb * 2 + (size_t)rows * 4;
    return *bytes <= (size_t)LDS_LIMIT;
}

static bool halo_shape_ok(const ConvArgs& a, int nb) {
    const bool square = a.kh == 3 && a.kw == 3;
    const bool line = (a.kh == 1 && (a.kw == 7 || a.kw == 3)) || (a.kw == 1 && (a.kh == 7 || a.kh == 3));
    if ((!square && !line) || a.sh != 1 || a.sw != 1 || a.pt != (a.kh - 1) / 2 || a.pl != (a.kw - 1) / 2) return false;
    if (a.Ho != a.H || a.Wo != a.W || a.pre_scale || a.cin % 32 || a.cout % 8) return false;
    // 32-bit byte offsets with 2^31 standing for 'outside'; float index arithmetic is exact below 2^24
    if ((long long)nb * a.H * a.W * a.x.stride * 2 >= 0x7FFFFF00LL || (long long)a.cout * a.kh * a.kw * a.cin * 2 >= 0x7FFFFF00LL) return false;
    if (halo_positions(a, nb) >= (1LL << 24)) return false;
    return true;
}

// Which variant runs this layer, -1: the generic kernel.  Measured on MI355X over the 3x3 layers
// of residual networks at batch 32 (56x56x64 to 7x7x512): the 128x64 tile with 64-channel blocks
// is the fastest or within 2 % of it everywhere; larger tiles lose more to the lower number of
// workgroups a compute unit can hold than they gain in traffic.  For the same reason a layer with
// several channel blocks and enough tiles to put more than two workgroups on every compute unit
// runs with one halo buffer (28x28x128: 27 us against 32, 14x14x256: 28 against 36).
int conv_halo_pick(const ConvArgs& a, int nb, int G) {
    if (!halo_shape_ok(a, nb)) return -1;
    int choice = -1;
    const long long PP = halo_positions(a, nb);
    const long long tiles = G * ((PP + 127) / 128) * ((a.cout + 63) / 64);
    if (a.kh != 3 || a.kw != 3) {
        // a one-dimensional filter: its four entries; one halo buffer under the same rule as below, and where two do not fit
        const int base = HALO_LINE + 4 * (a.kh == 1 ? (a.kw == 7 ? 0 : 2) : (a.kh == 7 ? 1 : 3)) + (a.cin % 64 == 0 ? 0 : 2);
        const bool one = a.cin > 64 && tiles > 2 * cu_budget();
        for (int k = one ? 1 : 0; k < 2; k++) {
            int hrows, nbuf;
            size_t bytes;
            const HaloVariant& v = HALO_VARIANTS[base + k];
            if (halo_layout(a, v, halo_splits(a, v, nb, G), &hrows, &nbuf, &bytes)) return base + k;
        }
        return -1;
    }
    if (a.cin % 64 == 0) {
        choice = a.cin > 64 && tiles > 2 * cu_budget() ? 6 : 0;
        // many tiles and whole 128-channel tiles: the wider tile reads two fragments per matrix-core instruction instead of three
        if (a.cin > 64 && a.cout % 128 == 0 && tiles / 2 >= 3 * cu_budget()) choice = 8;
        if (a.cout <= 32 && tiles > 2 * cu_budget()) choice = a.cin > 64 ? 12 : 13;   // narrow outputs (dense-block growth layers)
    } else if (a.cin >= 96) {
        choice = 4;                                              // multiples of 32 only: 32-channel blocks
    }
    if (choice < 0 || choice >= N_HALO_VARIANTS) return -1;
    int hrows, nbuf;
    size_t bytes;
    if (!halo_layout(a, HALO_VARIANTS[choice], halo_splits(a, HALO_VARIANTS[choice], nb, G), &hrows, &nbuf, &bytes)) return -1;
    return choice;
}

const char* conv_halo_name(int variant) { return HALO_VARIANTS[variant].name; }

template <int KH, int KW, int BP, int BC, int WP, int WC, int CB, int NHL>
static hipError_t launch_halo_variant(const ConvArgs& a, const ConvArgs* argv, int G, int nb, int splits, int hrows,
                                      int nbuf, size_t bytes, hipStream_t s) {
    static bool raised = false;                                  // LDS above 64 KB has to be asked for once
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void*)&conv_halo_bf16<KH, KW, BP, BC, WP, WC, CB, NHL>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_LIMIT);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const long long PP = halo_positions(a, nb);
    const dim3 grid((unsigned)(((PP + BP - 1) / BP) * ((a.cout + BC - 1) / BC)), splits, G);
    if (splits > 1) ENS_LAUNCH_FIRST((conv_halo_bf16<KH, KW, BP, BC, WP, WC, CB, NHL>), grid, dim3(256), bytes, s, argv, nb, hrows, nbuf);
    else ENS_LAUNCH((conv_halo_bf16<KH, KW, BP, BC, WP, WC, CB, NHL>), grid, dim3(256), bytes, s, argv, nb, hrows, nbuf);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && splits > 1) e = launch_conv_splitk_epilogue(a, argv, G, nb, nb * a.H * a.W, splits, s);
    return e;
}

hipError_t launch_conv_halo(const ConvArgs& a, const ConvArgs* argv, int G, int nb, int variant, hipStream_t s) {
    if (variant < 0 || variant >= N_HALO_VARIANTS || !halo_shape_ok(a, nb)) return hipErrorInvalidValue;
    if (a.x.stride % 8 || a.x.c0 % 8 || a.y.stride % 8 || a.y.c0 % 8) return hipErrorInvalidValue;
    if (a.res.p && (a.res.stride % 8 || a.res.c0 % 8)) return hipErrorInvalidValue;
    int hrows, nbuf;
    size_t bytes;
    int splits = halo_splits(a, HALO_VARIANTS[variant], nb, G);
    if (!halo_layout(a, HALO_VARIANTS[variant], splits, &hrows, &nbuf, &bytes)) return hipErrorInvalidValue;
    switch (variant) {
        case 0: return launch_halo_variant<3, 3, 128, 64, 2, 2, 64, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case 1: return launch_halo_variant<3, 3, 256, 64, 4, 1, 64, 2>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case 2: return launch_halo_variant<3, 3, 128, 128, 2, 2, 64, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case 3: return launch_halo_variant<3, 3, 256, 64, 4, 1, 32, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case 4: return launch_halo_variant<3, 3, 128, 64, 2, 2, 32, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case 5: return launch_halo_variant<3, 3, 128, 128, 2, 2, 32, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case 6: return launch_halo_variant<3, 3, 128, 64, 2, 2, 64, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case 7: return launch_halo_variant<3, 3, 256, 64, 4, 1, 64, 2>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case 8: return launch_halo_variant<3, 3, 128, 128, 2, 2, 64, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case 9: return launch_halo_variant<3, 3, 128, 64, 2, 2, 32, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case 10: return launch_halo_variant<3, 3, 256, 64, 4, 1, 32, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case 11: return launch_halo_variant<3, 3, 128, 128, 2, 2, 32, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case 12:
        case 13: return launch_halo_variant<3, 3, 256, 32, 4, 1, 64, 2>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case HALO_LINE + 0:
        case HALO_LINE + 1: return launch_halo_variant<1, 7, 128, 64, 2, 2, 64, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case HALO_LINE + 2:
        case HALO_LINE + 3: return launch_halo_variant<1, 7, 128, 64, 2, 2, 32, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case HALO_LINE + 4:
        case HALO_LINE + 5: return launch_halo_variant<7, 1, 128, 64, 2, 2, 64, 2>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case HALO_LINE + 6:
        case HALO_LINE + 7: return launch_halo_variant<7, 1, 128, 64, 2, 2, 32, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case HALO_LINE + 8:
        case HALO_LINE + 9: return launch_halo_variant<1, 3, 128, 64, 2, 2, 64, 2>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case HALO_LINE + 10:
        case HALO_LINE + 11: return launch_halo_variant<1, 3, 128, 64, 2, 2, 32, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case HALO_LINE + 12:
        case HALO_LINE + 13: return launch_halo_variant<3, 1, 128, 64, 2, 2, 64, 2>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        case HALO_LINE + 14:
        case HALO_LINE + 15: return launch_halo_variant<3, 1, 128, 64, 2, 2, 32, 1>(a, argv, G, nb, splits, hrows, nbuf, bytes, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ens
