// Device kernels of the ensemble library: argument blocks and host-side launchers.
// Every launcher validates what its kernel assumes and returns hipErrorInvalidValue
// instead of launching when a shape does not fit.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace ens {

typedef uint16_t bf16_t;   // raw bf16 bits in memory

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_SILU = 2 };

// A slice [c0, c0 + c) of the channels of an NHWC tensor whose pixels are `stride` elements apart.
struct View {
    void* p;
    int stride;
    int c0;
};

// Convolution (and its fused epilogue) over a batch of `nb` images.
//   y[n, ho, wo, co] = act( scale[co] * sum_{kh,kw,ci} pre(x[n, ho*sh-pt+kh, wo*sw-pl+kw, ci]) * w[co][kh][kw][ci]
//                           + bias[co] + res[n, ho, wo, co] )
// Weights are stored [cout][kh][kw][cin] (K contiguous per output channel).  The batch-norm that
// follows the convolution is scale (gamma / sqrt(var + eps)) and bias (beta - mean * scale + the
// layer's own bias * scale), both fp32 and applied to the fp32 sum: bf16 members keep the weights
// exactly as given (folding the scale into them would round every weight a second time, an error
// that is the same for all pixels of a channel and does not average out); fp32 members have the
// scale folded into the weights and a scale of ones.  pre_scale / pre_shift (fp32, per input
// channel) apply relu(x * scale + shift) to in-bounds inputs when non-null.
struct ConvArgs {
    View x, y, res;            // res.p == nullptr: no residual
    const void* w;
    const float* bias;         // never null (zeros when the layer has none)
    const float* scale;        // never null (ones when there is nothing to scale by)
    const float* pre_scale;
    const float* pre_shift;
    // split-K scratch of the worker (may be null: no splitting): room for ws_floats partial sums
    float* ws;
    long long ws_floats;
    const void* zeros;         // at least 16 bytes of zeros in device memory (padding source of the register-staged kernel)
    const void* wpk;           // the weights in matrix-core operand order (fused bottleneck kernel), or null
    // Squeeze-excite gate folded into a 1x1 convolution: input value (image n, channel ci) is multiplied by
    // gate[n * gate_stride + ci] (and rounded to bf16) before the matrix cores read it; null: no gate
    const float* gate;
    long long gate_stride;
    double inv_hw, inv_w;      // 1 / (Ho * Wo) and 1 / Wo, for the pixel index decomposition
    int nb, H, W, cin, Ho, Wo, cout;
    int kh, kw, sh, sw, pt, pl;
    int act;
};

struct PoolArgs {              // max / average pooling, depthwise convolution
    View x, y;
    const void* w;             // depthwise: [kh][kw][c] in the member's dtype
    const float* bias;         // depthwise only
    const float* scale;        // depthwise only: y = act(scale[c] * sum + bias[c]), as for ConvArgs
    int nb, H, W, c, Ho, Wo;
    int kh, kw, sh, sw, pt, pl;
    int act;
    // depthwise in front of a squeeze-excite block: each workgroup also leaves the channel sums of its outputs in the
    // block's scratch (per image `sums_stride` floats apart, one row of c floats per workgroup of the image), or null
    float* sums;
    int sums_stride;
    // average pool that runs in front of the pre-activated 1x1 convolution it stood behind: relu(x * pre_scale[c] +
    // pre_shift[c]) (fp32, per channel) is what it averages; null: the values as they are
    const float* pre_scale;
    const float* pre_shift;
};

struct GapArgs {               // global average pool to fp32 [nb][c]
    View x;
    float* y;
    const float* pre_scale;
    const float* pre_shift;
    int nb, HW, c;
};

struct FcArgs {                // logits[n][cout] = pooled[n][cin] . W[cin][cout] + bias
    const float* x;
    const void* w;             // [cin][cout] in the member's dtype
    const void* wpk;           // bf16 members: the transposed weights [cout][cin] in matrix-core operand order, or null
    const float* bias;
    float* y;                  // logits of the whole request, row stride ldy
    int nb, cin, cout;
    int64_t ldy;
};

// Squeeze-excite.  The channel sums of an image are taken by up to SE_MAX_SPLITS workgroups, each
// over a share of the pixels; the gate kernel adds their partial sums in a fixed order.
constexpr int SE_MAX_SPLITS = 16;
struct SeArgs {
    View x, y;
    const float* w1; const float* b1; const float* w2; const float* b2;   // fp32
    float* scratch;            // per image `cap` rows of c partial sums, r hidden values, c gates (floats)
    int nb, HW, c, r;
    int gate_only;             // non-zero: the gates go to `scratch` and y is not written (the consumer applies them)
    int cap;                   // rows of partial sums the scratch holds per image (SE_MAX_SPLITS, or more when the kernel
                               // that writes x leaves one row per workgroup)
    int have_sums;             // > 0: the kernel that wrote x has left this many rows of partial sums in `scratch`
};
// (the hidden values take a multiple of four floats: with c a multiple of four, every row stays 16-byte aligned)
__host__ __device__ inline int se_scratch_floats(int c, int r, int cap) { return (cap + 1) * c + (r + 3) / 4 * 4; }
__host__ __device__ inline int se_gate_offset(int c, int r, int cap) { return cap * c + (r + 3) / 4 * 4; }   // of an image's gates in its scratch
// Workgroups (of 256 lanes, one lane per 4 output columns x 8 channels) the summing depthwise kernel gives an image
__host__ __device__ inline int dwconv_sums_blocks(int Ho, int Wo, int c) { return (Ho * ((Wo + 3) / 4) * (c / 8) + 255) / 256; }

struct StageArgs {             // request images -> a worker's input tensor (convert, pad, resize)
    const float* src;          // request images, n x sh x sw x 3 fp32
    void* dst;                 // nb x dh x dw x dc, dtype of the member; see s2d
    int nb, sh, sw, dh, dw, dc;
    // s2d != 0 (bf16, dc == 16): the dh x dw image is stored "space to depth", as
    // ceil(dh/2) x ceil(dw/2) pixels whose channel (2*by + bx)*3 + c is channel c of image pixel
    // (2*r + by, 2*q + bx); channels 12..15 and pixels past the image are zero.  A stride-2
    // convolution over the image is a stride-1 convolution over this tensor.
    int s2d;
};

// Every launcher runs one kernel for a gang of G members that execute the same operation on
// tensors of the same shape (the co-located replicas of a homogeneous ensemble): argv is a device
// array of G argument blocks, blockIdx.z picks the member, `a` is the host copy of argv[0] used
// for validation and grid sizing.  nb is the number of images of this batch; `first` is the index
// of the batch's first image in the request (input staging reads there, the FC head writes there).
hipError_t launch_conv_bf16(const ConvArgs& a, const ConvArgs* argv, int G, int nb, hipStream_t s);
hipError_t launch_conv_f32(const ConvArgs& a, const ConvArgs* argv, int G, int nb, hipStream_t s);
hipError_t launch_dwconv(const PoolArgs& a, const PoolArgs* argv, int G, int nb, bool bf16, hipStream_t s);
bool dwconv_sums_applicable(const PoolArgs& a, bool bf16);     // can the depthwise kernel also leave the channel sums of its output?
hipError_t launch_pool(const PoolArgs& a, const PoolArgs* argv, int G, int nb, bool is_max, bool bf16, hipStream_t s);
hipError_t launch_gap(const GapArgs& a, const GapArgs* argv, int G, int nb, bool bf16, hipStream_t s);
hipError_t launch_fc(const FcArgs& a, const FcArgs* argv, int G, int nb, long long first, bool bf16, hipStream_t s);
// the FC head on the matrix cores (bf16 members with a packed weight copy); launch_fc takes it when it applies
bool fc_mfma_applicable(const FcArgs& a);
hipError_t launch_fc_mfma(const FcArgs& a, const FcArgs* argv, int G, int nb, long long first, hipStream_t s);
hipError_t launch_se(const SeArgs& a, const SeArgs* argv, int G, int nb, bool bf16, hipStream_t s);
hipError_t launch_stage(const StageArgs& a, const StageArgs* argv, int G, int nb, long long first, bool bf16, hipStream_t s);
// Combination rule; logits: n_members pointers (device array).
//   COMBINE_MEAN      Y[i, :] = sum_m softmax(logits_m[i, :]) / M
//   COMBINE_WEIGHTED  Y[i, :] = sum_m weights[m] * softmax(logits_m[i, :])   (weights: device, n_members floats)
//   COMBINE_VOTE      Y[i, c] = #{m : argmax logits_m[i, :] == c} / M        (lowest index on exact ties)
enum { COMBINE_MEAN = 0, COMBINE_WEIGHTED = 1, COMBINE_VOTE = 2 };
hipError_t launch_combine(const float* const* logits, const float* weights, int rule, int n_members, int64_t n,
                          int classes, float* y, hipStream_t s);
hipError_t launch_fill_noise(float* p, int64_t count, uint64_t seed, hipStream_t s);
hipError_t launch_fill_zero(float* p, int64_t count, hipStream_t s);

double conv_flops(const ConvArgs& a, int nb);

// Per-kernel timing.  Events put here are attached to the dispatch of the next kernel this thread
// launches: the runtime stamps `start` with the begin of that kernel and `stop` with its end, with
// no extra packet in the stream (an event recorded before and after a launch also measures the gap
// between the two packets).  A launcher that issues several kernels gives `start` to the first
// and `stop` to the last.  Null: no timing.
struct LaunchEvents {
    hipEvent_t start = nullptr, stop = nullptr;
};
LaunchEvents& next_launch_events();                  // per thread

// Compute units a launch may count on: all 256 when its stream has the GPU to itself, a share of them
// when several worker streams run at once.  The launchers' tile and split choices weigh idle compute
// units against efficiency per workgroup by this number; the engine sets it (per thread) to the chip's
// units divided by the number of streams of the installed allocation.
int& cu_budget();

}  // namespace ens

// The only, first, middle and last kernel of a launcher.
#define ENS_LAUNCH_EV(take_start, take_stop, kernel, grid, block, shmem, stream, ...)                            \
    do {                                                                                                          \
        ens::LaunchEvents& nle_ = ens::next_launch_events();                                                      \
        hipEvent_t ev_start_ = (take_start) ? nle_.start : nullptr, ev_stop_ = (take_stop) ? nle_.stop : nullptr; \
        if (take_start) nle_.start = nullptr;                                                                     \
        if (take_stop) nle_.stop = nullptr;                                                                       \
        hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, ev_start_, ev_stop_, 0, __VA_ARGS__);           \
    } while (0)
#define ENS_LAUNCH(kernel, grid, block, shmem, stream, ...) ENS_LAUNCH_EV(true, true, kernel, grid, block, shmem, stream, __VA_ARGS__)
#define ENS_LAUNCH_FIRST(kernel, grid, block, shmem, stream, ...) ENS_LAUNCH_EV(true, false, kernel, grid, block, shmem, stream, __VA_ARGS__)
#define ENS_LAUNCH_MIDDLE(kernel, grid, block, shmem, stream, ...) ENS_LAUNCH_EV(false, false, kernel, grid, block, shmem, stream, __VA_ARGS__)
#define ENS_LAUNCH_LAST(kernel, grid, block, shmem, stream, ...) ENS_LAUNCH_EV(false, true, kernel, grid, block, shmem, stream, __VA_ARGS__)
