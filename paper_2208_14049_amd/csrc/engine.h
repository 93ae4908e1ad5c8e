// The inference-system core on one GPU: members resident in HBM, workers (one per non-zero
// cell of the allocation matrix) with their own stream and activation arena, the segment /
// batch partition of a request and the fused combination kernel.
#pragma once
#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "../../include/ens.h"
#include "kernels.h"

namespace ens {

struct TensorInfo {
    int h, w, c;
    int cs;          // stored channels (bf16 tensors are padded to a multiple of 8)
    bool f32;        // stored as fp32
    int def, last;   // first writing / last reading operation (-1: written by the input staging)
    bool external;   // the logits tensor lives in the member's logits buffer, not in an arena
    size_t elems_per_image() const { return (size_t)h * w * cs; }
    size_t bytes(int batch) const { return (size_t)batch * elems_per_image() * (f32 ? 4 : 2); }
};

struct OpPlan {
    ens_op op;
    // byte offsets into the member's device parameter block (SIZE_MAX: absent)
    size_t w, b, scale, pre_scale, pre_shift, w2, b2;
    size_t w_packed; // the convolution's weights once more in matrix-core operand order (members of a fused chain)
    int cin_s;       // stored input channels of the convolution's K axis
    int scratch;     // index of the scratch pseudo-tensor (squeeze-excite), -1 otherwise
    int alg_k;       // multiply-adds per output element as the network defines the layer (0: kh*kw*cin of op)
    // A grouped convolution runs as `sub` dense convolutions on channel slices, sub_cout output channels
    // each over cin_s input channels, weights [sub][sub_cout][kh*kw][cin_s] (zeros where a pair of
    // channels belongs to different groups).  Ordinary convolution: sub = 1, sub_cout = cout.
    int sub, sub_cout;
    // This convolution and the next one read the same input slice and write outputs of the same height
    // and width (a residual block's 3x3 / stride-2 branch and its 1x1 shortcut, the 1x1 heads of an
    // inception module's branches): one launch can run both as further argument blocks when both go
    // to the generic kernel.  The second output counts as written here.
    bool fuse_next;
    // This 1x1 convolution, the 3x3 after it and the 1x1 after that form a residual bottleneck whose two
    // middle tensors nobody else touches: one kernel can run the three without writing them.
    bool fuse_chain;
    // This pre-activated 1x1 convolution (to 128 channels) and the 3x3 after it (to 32 channels) are a layer
    // of a dense block whose middle tensor nobody else touches: one kernel can run both.
    bool fuse_dense;
    // This convolution is the input stem (rewritten to stride 1 over the space-to-depth image, ReLU) and the
    // next operation is a 3x3 / stride-2 / padding-1 max-pool that alone reads its output: one kernel can
    // run both without writing the stem's output.
    bool fuse_pool;
    // This squeeze-excite block is followed by a 1x1 convolution that alone reads its output: the block can
    // stop at the gates and the convolution multiply its input by them, so that the rescaled tensor is
    // never written.
    bool fuse_gate;
    // This depthwise convolution is followed by a squeeze-excite block over its output: its kernel can leave
    // the channel sums the block starts from (one row per workgroup, in the block's scratch, which then lives
    // from this operation on and holds se_cap rows), and the block does not read the tensor for them.
    bool fuse_sums;
    // This 3x3 / stride-1 / padding-1 average pool is followed by a plain 1x1 convolution that alone reads its output
    // and has no more output channels than the pool has channels (the pool branch of an inception module): the
    // two are linear and commute, so the convolution (with its batch-norm, which an average whose weights add up
    // to one also commutes with) can run first, into the pool's output memory, and the pool then averages the
    // narrower tensor and applies the activation.
    bool swap_pool;
    // This pre-activated 1x1 convolution without an activation of its own is followed by a 2x2 / stride-2 average
    // pool that alone reads its output (the transition between two dense blocks): pre-activation and pool can run
    // first, into the convolution's output memory, and the convolution on a quarter of the pixels.
    bool swap_conv;
    int se_cap;      // squeeze-excite: rows of partial sums its scratch holds per image
};

struct Member {
    bool bf16 = false;
    int in_h = 0, in_w = 0, classes = 0, out_tensor = -1;
    std::vector<TensorInfo> tensors;     // description tensors, then scratch pseudo-tensors
    std::vector<OpPlan> ops;
    std::vector<uint8_t> host_params;    // folded, converted, laid out for the device
    size_t zeros_off = 0;                // 256 zero bytes inside the parameter block (padding source)
    // The stride-2 convolution that reads the input image runs as a stride-1 convolution over the
    // image stored space-to-depth (tensor 0 is then ceil(h/2) x ceil(w/2) x 12, stored 16 wide).
    bool stem_s2d = false;
    char* dev_params = nullptr;
    size_t weight_bytes() const { return host_params.size(); }
};

// Scratch the convolution kernel uses when it splits a layer's K range over several workgroups:
// one fp32 slice of partial sums per split.
constexpr size_t SPLIT_WS_FLOATS = 4u << 20;

struct ArenaLayout {
    std::vector<size_t> offset;          // per tensor (unused for external ones)
    size_t scratch_offset = SIZE_MAX;    // split-K scratch (bf16 members)
    size_t bytes = 0;
};

// Builds the device-side form of a member from its description.  Host only.
int build_member(const ens_member_spec& spec, const float* params, Member* out);
// Places the member's tensors for `batch` images by liveness; host only.
// keep_all gives every tensor its own region (debug read-back of intermediate tensors).
ArenaLayout plan_arena(const Member& m, int batch, bool keep_all = false);

enum LaunchKind { L_CONV, L_DWCONV, L_POOL, L_GAP, L_FC, L_SE, L_BNECK, L_DENSE, L_STEMPOOL, L_SKIP };   // L_SKIP: ran with an earlier launch

// One operation of a gang: host copy of the first member's arguments (validation, grid sizing)
// and the device array holding the arguments of every member of the gang.
struct Launch {
    int kind = 0;
    bool is_max = false;
    int klass = 0;                 // profile class
    double flop = 0, bytes = 0;    // algorithmic work of one member's full-batch launch
    ConvArgs conv;
    ConvArgs conv2, conv3;         // L_BNECK: the second and third convolution of the chain; L_DENSE: conv2 is the 3x3;
                                   // L_STEMPOOL: conv2 describes the pooled output
    PoolArgs pool;
    GapArgs gap;
    FcArgs fc;
    SeArgs se;
    const void* d_argv = nullptr;  // device: G * sub argument blocks of this operation's kind
    int sub = 1;                   // argument blocks per member (sub-convolutions of a grouped convolution)
};

struct Worker {
    int member = 0, batch = 0, slot = 0;
    int rank = 0, of = 1;          // this is worker `rank` of the member's `of` workers
    int gang = -1;
    char* arena = nullptr;
    size_t arena_bytes = 0;
    ArenaLayout layout;
    int last_nb = 0;
};

// Workers that run the same network shape at the same batch size on the same segments (the
// replicas of a homogeneous ensemble in one row of the allocation matrix) advance in lockstep:
// one stream, and one kernel launch per operation whose grid spans all of them.
struct Gang {
    std::vector<int> workers;      // indices into ens_handle::workers; [0] leads (its input tensor is shared)
    int rank = 0, of = 1;
    hipStream_t stream = nullptr;
    hipEvent_t done = nullptr;
    std::vector<Launch> launches;
    StageArgs stage;
    const StageArgs* d_stage = nullptr;
    char* d_args = nullptr;        // device block holding every argument array of the gang
    size_t d_args_bytes = 0;
};

struct ProfClass {
    std::string name;
    double ms = 0, flop = 0, bytes = 0;
    int64_t launches = 0;
};

struct ProfRec { int klass; hipEvent_t start, stop; double flop, bytes; };

}  // namespace ens

struct ens_handle {
    std::vector<ens::Member> members;
    std::vector<ens::Worker> workers;
    std::vector<ens::Gang> gangs;
    bool gangs_enabled = true;                   // false: every worker is a gang of its own
    bool args_stale = false;                     // request buffers moved: argument arrays need rebuilding
    ens_alloc alloc;
    bool have_alloc = false;
    int segment_size = 128;
    int base_h = 0, base_w = 0, classes = 0;
    bool images_on_device = false, probs_on_device = false;
    uint64_t budget = 0;                         // 0: whatever the device has
    hipStream_t main_stream = nullptr;
    hipEvent_t input_ready = nullptr;
    // request buffers, grown on demand
    float* d_images = nullptr;  size_t d_images_cap = 0;
    float* d_probs = nullptr;   size_t d_probs_cap = 0;
    // Per-member logits of the request in flight.  d_logits / d_logit_table are the buffers in use:
    // either the library's own allocations (d_logits_heap, d_logit_ptrs; grown on demand) or, for the
    // allocation-free entry point, slices of the fixed device array.
    std::vector<float*> d_logits; size_t d_logits_rows = 0;      // in use, and the rows they hold
    std::vector<float*> d_logits_heap; size_t d_logits_heap_rows = 0;
    const float** d_logit_ptrs = nullptr;                        // device table of the heap pointers
    const float** d_logit_table = nullptr;                       // device table of the pointers in use
    bool logits_static = false;
    int combine_rule = 0;                        // ENS_COMBINE_*
    float* d_weights = nullptr;                  // member weights of the weighted rule (device)
    float* d_calib = nullptr;   size_t d_calib_images = 0;
    const float* bound_images = nullptr;         // request images the staging arguments point at
    int stage_klass = 0;
    int64_t last_n = 0;
    double last_ms = 0;
    // profiling
    bool profiling = false;
    bool keep_tensors = false;                   // debug: no reuse of arena regions
    bool fake_predictor = false;                 // overhead experiment: forward passes replaced by zeros
    bool one_stream = false;                     // measurement: every worker issues on the main stream, one kernel at a time
    std::vector<ens::ProfClass> prof;
    std::vector<ens::ProfRec> prof_recs;
    std::vector<hipEvent_t> event_pool;
};
