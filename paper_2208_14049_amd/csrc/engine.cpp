// The inference-system core (section "The inference system") on one GPU and its C interface.
//
// The paper's processes become: the segment broadcaster -> a host loop that hands every segment
// once to every member; a worker (batcher, predictor, prediction sender) -> a HIP stream plus an
// activation arena whose kernels write logits straight into the member's row block, so there
// is nothing to reassemble; the prediction accumulator -> one fused softmax-and-mean kernel
// after an event join of all worker streams (fixed member order, no atomics).
#include "engine.h"

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstring>

#include "planner.h"
#include "seedgen.h"
#include "static_scratch.h"

using namespace ens;

#define HIP_TRY(expr)                                                                       \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) {                                                             \
            fprintf(stderr, "ens: %s failed: %s (%s:%d)\n", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return e_ == hipErrorOutOfMemory ? ENS_E_NOMEM : ENS_E_HIP;                     \
        }                                                                                   \
    } while (0)

namespace ens {

const char* conv_bf16_variant_name(const ConvArgs& a, int G);
bool conv_bneck_applicable(const ConvArgs& a1, const ConvArgs& a2, const ConvArgs& a3, int nb, int G);
const char* conv_bneck_name(const ConvArgs& a1);
hipError_t launch_conv_bneck(const ConvArgs& a1, const ConvArgs& a2, const ConvArgs& a3, const ConvArgs* argv, int G, int nb,
                             hipStream_t s);
bool conv_dense_applicable(const ConvArgs& a1, const ConvArgs& a2, int nb, int G);
bool conv_pw_applicable(const ConvArgs& a, int nb, int G);
bool conv_stempool_applicable(const ConvArgs& a, const ConvArgs& pool, int nb, int G);
const char* conv_stempool_name();
hipError_t launch_conv_stempool(const ConvArgs& a, const ConvArgs& pool, const ConvArgs* argv, int G, int nb, hipStream_t s);
const char* conv_dense_name();
hipError_t launch_conv_dense(const ConvArgs& a1, const ConvArgs& a2, const ConvArgs* argv, int G, int nb, hipStream_t s);

static int prof_class(ens_handle* h, const std::string& name) {
    for (size_t i = 0; i < h->prof.size(); i++)
        if (h->prof[i].name == name) return (int)i;
    h->prof.push_back(ProfClass{name});
    return (int)h->prof.size() - 1;
}

// Tensor 0 (the staged input) is shared by a gang: only the leader's copy is written.
static View view_of(const Worker& w, const Worker& leader, const Member& m, int t, int c0) {
    const Worker& src = t == 0 ? leader : w;
    View v;
    v.p = src.arena + src.layout.offset[t];
    v.stride = m.tensors[t].cs;
    v.c0 = c0;
    return v;
}

static bool same_network(const Member& a, const Member& b) {
    if (a.bf16 != b.bf16 || a.ops.size() != b.ops.size() || a.tensors.size() != b.tensors.size()) return false;
    for (size_t t = 0; t < a.tensors.size(); t++)
        if (a.tensors[t].h != b.tensors[t].h || a.tensors[t].w != b.tensors[t].w || a.tensors[t].c != b.tensors[t].c) return false;
    for (size_t i = 0; i < a.ops.size(); i++)
        if (memcmp(&a.ops[i].op, &b.ops[i].op, sizeof(ens_op)) != 0) return false;
    return true;
}

// Fills one member's argument block for operation `pl`; `L` receives kind, class and work.
// `sub`: which of the operation's pl.sub argument blocks (sub-convolutions of a grouped convolution)
static int fill_args(ens_handle* h, const Worker& w, const Worker& leader, int G, const OpPlan& pl, Launch& L, int sub = 0) {
    const Member& m = h->members[w.member];
    const int es = m.bf16 ? 2 : 4;
    const ens_op& o = pl.op;
    const TensorInfo& ts = m.tensors[o.src];
    const TensorInfo& td = m.tensors[o.dst];
    const char* P = m.dev_params;
    const double nb = w.batch;
    switch (o.kind) {
        case ENS_OP_CONV: {
            L.kind = L_CONV;
            ConvArgs& a = L.conv;
            a.x = view_of(w, leader, m, o.src, o.src_c0);
            a.y = view_of(w, leader, m, o.dst, o.dst_c0);
            a.res.p = nullptr; a.res.stride = 0; a.res.c0 = 0;
            if (o.res >= 0) a.res = view_of(w, leader, m, o.res, o.res_c0);
            a.w = P + pl.w;
            a.bias = (const float*)(P + pl.b);
            a.scale = (const float*)(P + pl.scale);
            a.pre_scale = pl.pre_scale != SIZE_MAX ? (const float*)(P + pl.pre_scale) : nullptr;
            a.pre_shift = pl.pre_shift != SIZE_MAX ? (const float*)(P + pl.pre_shift) : nullptr;
            a.ws = nullptr; a.ws_floats = 0;
            a.gate = nullptr; a.gate_stride = 0;
            a.zeros = P + m.zeros_off;
            a.wpk = pl.w_packed != SIZE_MAX ? P + pl.w_packed : nullptr;
            if (w.layout.scratch_offset != SIZE_MAX) {
                a.ws = (float*)(w.arena + w.layout.scratch_offset);
                a.ws_floats = (long long)SPLIT_WS_FLOATS;
            }
            a.nb = w.batch; a.H = ts.h; a.W = ts.w; a.cin = pl.cin_s; a.Ho = td.h; a.Wo = td.w; a.cout = pl.sub_cout;
            a.kh = o.kh; a.kw = o.kw; a.sh = o.sh; a.sw = o.sw; a.pt = o.pt; a.pl = o.pl; a.act = o.act;
            a.inv_hw = 1.0 / ((double)td.h * td.w); a.inv_w = 1.0 / (double)td.w;
            L.sub = pl.sub;
            if (pl.sub > 1) {                                    // this block's slice of channels, weights and bias
                a.x.c0 += sub * pl.cin_s;
                a.y.c0 += sub * pl.sub_cout;
                if (a.res.p) a.res.c0 += sub * pl.sub_cout;
                a.w = (const char*)a.w + (size_t)sub * pl.sub_cout * o.kh * o.kw * pl.cin_s * es;
                a.bias += (size_t)sub * pl.sub_cout;
                a.scale += (size_t)sub * pl.sub_cout;
            }
            const int groups = o.r > 1 ? o.r : 1;
            L.flop = 2.0 * nb * td.h * td.w * o.cout * (pl.alg_k > 0 ? pl.alg_k : o.kh * o.kw * o.cin / groups);
            L.bytes = nb * ((double)ts.h * ts.w * o.cin + (double)td.h * td.w * o.cout * (o.res >= 0 ? 2 : 1)) * es +
                      (double)o.kh * o.kw * o.cin / groups * o.cout * es;
            L.klass = prof_class(h, m.bf16 ? conv_bf16_variant_name(a, G * pl.sub) : "conv_f32_kernel");
            break;
        }
        case ENS_OP_DWCONV:
        case ENS_OP_MAXPOOL:
        case ENS_OP_AVGPOOL: {
            L.kind = o.kind == ENS_OP_DWCONV ? L_DWCONV : L_POOL;
            L.is_max = o.kind == ENS_OP_MAXPOOL;
            PoolArgs& a = L.pool;
            a.x = view_of(w, leader, m, o.src, o.src_c0);
            a.y = view_of(w, leader, m, o.dst, o.dst_c0);
            a.w = o.kind == ENS_OP_DWCONV ? P + pl.w : nullptr;
            a.bias = o.kind == ENS_OP_DWCONV ? (const float*)(P + pl.b) : nullptr;
            a.scale = o.kind == ENS_OP_DWCONV ? (const float*)(P + pl.scale) : nullptr;
            a.nb = w.batch; a.H = ts.h; a.W = ts.w; a.c = o.cin; a.Ho = td.h; a.Wo = td.w;
            a.kh = o.kh; a.kw = o.kw; a.sh = o.sh; a.sw = o.sw; a.pt = o.pt; a.pl = o.pl;
            a.act = o.kind == ENS_OP_DWCONV ? o.act : ACT_NONE;  // a pool has none of its own
            a.sums = nullptr; a.sums_stride = 0;
            a.pre_scale = a.pre_shift = nullptr;
            L.flop = o.kind == ENS_OP_DWCONV ? 2.0 * nb * td.h * td.w * o.cin * o.kh * o.kw : 0.0;
            L.bytes = nb * ((double)ts.h * ts.w + (double)td.h * td.w) * o.cin * es;
            L.klass = prof_class(h, o.kind == ENS_OP_DWCONV ? "window_kernel<dwconv>"
                                    : L.is_max ? "window_kernel<maxpool>" : "window_kernel<avgpool>");
            break;
        }
        case ENS_OP_GAP: {
            L.kind = L_GAP;
            GapArgs& a = L.gap;
            a.x = view_of(w, leader, m, o.src, o.src_c0);
            a.y = (float*)(w.arena + w.layout.offset[o.dst]) + o.dst_c0;
            a.pre_scale = pl.pre_scale != SIZE_MAX ? (const float*)(P + pl.pre_scale) : nullptr;
            a.pre_shift = pl.pre_shift != SIZE_MAX ? (const float*)(P + pl.pre_shift) : nullptr;
            a.nb = w.batch; a.HW = ts.h * ts.w; a.c = o.cin;
            if (td.c != o.cin) return ENS_E_UNSUPPORTED;         // the pooled vector is dense
            L.bytes = nb * (double)ts.h * ts.w * o.cin * es;
            L.klass = prof_class(h, "gap_kernel");
            break;
        }
        case ENS_OP_FC: {
            L.kind = L_FC;
            FcArgs& a = L.fc;
            a.x = (const float*)(w.arena + w.layout.offset[o.src]);
            a.w = P + pl.w;
            a.wpk = pl.w_packed != SIZE_MAX ? P + pl.w_packed : nullptr;
            a.bias = (const float*)(P + pl.b);
            a.y = h->d_logits[w.member];                         // rows of the whole request
            a.nb = w.batch; a.cin = o.cin; a.cout = o.cout; a.ldy = o.cout;
            L.flop = 2.0 * nb * o.cin * o.cout;
            L.bytes = (double)o.cin * o.cout * es + nb * (o.cin + o.cout) * 4.0;
            L.klass = prof_class(h, m.bf16 && fc_mfma_applicable(a) ? "fc_mfma_bf16" : "fc_kernel");
            break;
        }
        case ENS_OP_SE: {
            L.kind = L_SE;
            SeArgs& a = L.se;
            a.x = view_of(w, leader, m, o.src, o.src_c0);
            a.y = view_of(w, leader, m, o.dst, o.dst_c0);
            a.w1 = (const float*)(P + pl.w); a.b1 = (const float*)(P + pl.b);
            a.w2 = (const float*)(P + pl.w2); a.b2 = (const float*)(P + pl.b2);
            a.scratch = (float*)(w.arena + w.layout.offset[pl.scratch]);
            a.nb = w.batch; a.HW = ts.h * ts.w; a.c = o.cin; a.r = o.r;
            a.gate_only = 0;
            a.cap = pl.se_cap; a.have_sums = 0;
            L.flop = 4.0 * nb * o.cin * o.r;
            L.bytes = nb * 3.0 * ts.h * ts.w * o.cin * es;
            L.klass = prof_class(h, "se_kernels");
            break;
        }
        default:
            return ENS_E_INVALID;
    }
    return ENS_OK;
}

// Translates the gang's operations into kernel argument arrays in device memory.
// may_alloc false: the device block of the gang must already be large enough (it is once the
// allocation has been installed); the function then only rewrites it.
static int build_launches(ens_handle* h, Gang& g, bool may_alloc = true) {
    const Worker& leader = h->workers[g.workers[0]];
    const Member& m = h->members[leader.member];
    const int G = (int)g.workers.size();
    const size_t slot = 512;                                     // bytes reserved per argument block
    static_assert(sizeof(ConvArgs) <= 512 && sizeof(PoolArgs) <= 512 && sizeof(SeArgs) <= 512, "argument block");
    // Which bottlenecks run as one kernel: planned as such and within the kernel's shapes at this batch
    // size.  The tensors in between are then not written (not wanted when they are to be read back).
    std::vector<char> chain(m.ops.size(), 0);                    // 1: runs the next two operations too, 2: run by it
    for (size_t i = 0; i + 2 < m.ops.size(); i++) {
        if (!m.ops[i].fuse_chain || h->keep_tensors) continue;
        Launch a, b, c;
        if (fill_args(h, leader, leader, G, m.ops[i], a) != ENS_OK || fill_args(h, leader, leader, G, m.ops[i + 1], b) != ENS_OK ||
            fill_args(h, leader, leader, G, m.ops[i + 2], c) != ENS_OK)
            continue;
        if (conv_bneck_applicable(a.conv, b.conv, c.conv, leader.batch, G)) {
            chain[i] = 1;
            chain[i + 1] = chain[i + 2] = 2;
        }
    }
    // Which layers of dense blocks run as one kernel: chain[] 3 marks the head (two operations), 2 the one it runs
    for (size_t i = 0; i + 1 < m.ops.size(); i++) {
        if (!m.ops[i].fuse_dense || h->keep_tensors || chain[i] || chain[i + 1]) continue;
        Launch a, b;
        if (fill_args(h, leader, leader, G, m.ops[i], a) != ENS_OK || fill_args(h, leader, leader, G, m.ops[i + 1], b) != ENS_OK) continue;
        if (conv_dense_applicable(a.conv, b.conv, leader.batch, G)) {
            chain[i] = 3;
            chain[i + 1] = 2;
        }
    }
    // The stem and the max-pool behind it as one kernel: chain[] 4 marks the stem, 2 the pool it runs
    auto pool_as_conv = [&](const Worker& w, const OpPlan& pl) {   // the pooled output in the convolution's argument form
        const Member& mw = h->members[w.member];
        ConvArgs p;
        memset(&p, 0, sizeof(p));
        p.y = view_of(w, leader, mw, pl.op.dst, pl.op.dst_c0);
        p.Ho = mw.tensors[pl.op.dst].h;
        p.Wo = mw.tensors[pl.op.dst].w;
        p.nb = w.batch;
        return p;
    };
    for (size_t i = 0; i + 1 < m.ops.size(); i++) {
        if (!m.ops[i].fuse_pool || h->keep_tensors || chain[i] || chain[i + 1]) continue;
        Launch a;
        if (fill_args(h, leader, leader, G, m.ops[i], a) != ENS_OK) continue;
        if (conv_stempool_applicable(a.conv, pool_as_conv(leader, m.ops[i + 1]), leader.batch, G)) {
            chain[i] = 4;
            chain[i + 1] = 2;
        }
    }
    // Which pairs of convolutions run as one launch: planned as such, and both on the generic kernel
    // for this batch size (its workgroups read every field of their own argument block).
    std::vector<char> fused(m.ops.size(), 0);                    // 1: takes the next operation along, 2: taken along
    for (size_t i = 0; i + 1 < m.ops.size(); i++) {
        if (!m.ops[i].fuse_next || chain[i] || chain[i + 1]) continue;   // a bottleneck kernel takes precedence
        Launch a, b;
        if (fill_args(h, leader, leader, G, m.ops[i], a) != ENS_OK || fill_args(h, leader, leader, G, m.ops[i + 1], b) != ENS_OK) continue;
        a.conv.wpk = b.conv.wpk = nullptr;                       // a pair runs on the generic kernel
        const char* generic = "conv_igemm_bf16";
        if (strncmp(conv_bf16_variant_name(a.conv, 2 * G), generic, strlen(generic)) == 0 &&
            strncmp(conv_bf16_variant_name(b.conv, 2 * G), generic, strlen(generic)) == 0) {
            fused[i] = 1;
            fused[i + 1] = 2;
        }
    }
    // Squeeze-excite blocks that stop at the gates, which the 1x1 convolution behind them applies to its
    // input: gated[] 1 marks the block, 2 the convolution.  gate_args turns the convolution's arguments round.
    std::vector<char> gated(m.ops.size(), 0);
    auto gate_args = [&](const Worker& w, const OpPlan& se, ConvArgs& c) {
        const Member& mw = h->members[w.member];
        c.x = view_of(w, leader, mw, se.op.src, se.op.src_c0);
        c.gate = (const float*)(w.arena + w.layout.offset[se.scratch]) + se_gate_offset(se.op.cin, se.op.r, se.se_cap);
        c.gate_stride = se_scratch_floats(se.op.cin, se.op.r, se.se_cap);
    };
    for (size_t i = 0; i + 1 < m.ops.size(); i++) {
        if (!m.ops[i].fuse_gate || h->keep_tensors || chain[i] || chain[i + 1] || fused[i] || fused[i + 1]) continue;
        Launch c;
        if (fill_args(h, leader, leader, G, m.ops[i + 1], c) != ENS_OK) continue;
        gate_args(leader, m.ops[i], c.conv);
        if (c.conv.wpk && conv_pw_applicable(c.conv, leader.batch, G)) {
            gated[i] = 1;
            gated[i + 1] = 2;
        }
    }
    // Depthwise convolutions whose kernel leaves the channel sums for the squeeze-excite block behind them:
    // summed[] 1 marks the convolution, 2 the block.
    std::vector<char> summed(m.ops.size(), 0);
    for (size_t i = 0; i + 1 < m.ops.size(); i++) {
        if (!m.ops[i].fuse_sums || h->keep_tensors || m.ops[i + 1].op.kind != ENS_OP_SE) continue;
        Launch d;
        if (fill_args(h, leader, leader, G, m.ops[i], d) != ENS_OK) continue;
        if (dwconv_sums_applicable(d.pool, m.bf16) && dwconv_sums_blocks(d.pool.Ho, d.pool.Wo, d.pool.c) <= m.ops[i + 1].se_cap) {
            summed[i] = 1;
            summed[i + 1] = 2;
        }
    }
    // Average pools that change places with the 1x1 convolution behind them: swapped[] 1 marks the pool's place
    // (the convolution runs there), 2 the convolution's (the pool runs there, on the convolution's channels).
    std::vector<char> swapped(m.ops.size(), 0);
    for (size_t i = 0; i + 1 < m.ops.size(); i++) {
        if (!m.ops[i].swap_pool || h->keep_tensors || chain[i] || chain[i + 1] || fused[i] || fused[i + 1] || gated[i + 1]) continue;
        swapped[i] = 1;
        swapped[i + 1] = 2;
    }
    // ... and pre-activated 1x1 convolutions that let the 2x2 average pool behind them go first: 3 marks the
    // convolution's place (the pool runs there, on the convolution's input), 4 the pool's (the convolution, on the pooled map)
    for (size_t i = 0; i + 1 < m.ops.size(); i++) {
        if (!m.ops[i].swap_conv || h->keep_tensors || chain[i] || chain[i + 1] || fused[i] || fused[i + 1] || gated[i] || swapped[i] ||
            swapped[i + 1])
            continue;
        swapped[i] = 3;
        swapped[i + 1] = 4;
    }
    std::vector<size_t> first_blk(m.ops.size() + 1, 0);          // argument blocks: G * sub per operation
    for (size_t i = 0; i < m.ops.size(); i++)
        first_blk[i + 1] = first_blk[i] + (fused[i] == 2 || chain[i] == 2 ? 0
                                           : (size_t)G * (chain[i] == 1 ? 3 : chain[i] == 3 || chain[i] == 4 || fused[i] == 1 ? 2 : (m.ops[i].sub > 1 ? m.ops[i].sub : 1)));
    const size_t n_blk = first_blk[m.ops.size()];
    std::vector<char> host((n_blk + (size_t)G) * slot, 0);
    if (!may_alloc && (!g.d_args || g.d_args_bytes < host.size())) return ENS_E_INVALID;
    if (g.d_args && g.d_args_bytes < host.size()) { (void)hipFree(g.d_args); g.d_args = nullptr; }
    if (!g.d_args) { HIP_TRY(hipMalloc((void**)&g.d_args, host.size())); g.d_args_bytes = host.size(); }
    g.launches.clear();
    for (size_t i = 0; i < m.ops.size(); i++) {
        Launch L;
        if (fused[i] == 2 || chain[i] == 2) {                    // its argument blocks are in an earlier launch
            L.kind = L_SKIP;
            g.launches.push_back(L);
            continue;
        }
        if (chain[i] == 4) {                                     // stem and pool: G blocks of the convolution, then G of the pooled output
            for (int k = G - 1; k >= 0; k--) {
                const Worker& wk = h->workers[g.workers[k]];
                const Member& mk = h->members[wk.member];
                const ConvArgs p = pool_as_conv(wk, mk.ops[i + 1]);
                const int rc = fill_args(h, wk, leader, G, mk.ops[i], L);
                if (rc != ENS_OK) return rc;
                L.conv.ws = nullptr;
                L.conv.ws_floats = 0;
                if (k == 0) L.conv2 = p;
                memcpy(host.data() + (first_blk[i] + (size_t)k) * slot, &L.conv, sizeof(ConvArgs));
                memcpy(host.data() + (first_blk[i] + (size_t)G + k) * slot, &p, sizeof(ConvArgs));
            }
            // algorithmic bytes: the image once, the pooled map once, the filter
            L.bytes = (double)leader.batch * ((double)L.conv.H * L.conv.W * L.conv.cin + (double)L.conv2.Ho * L.conv2.Wo * L.conv.cout) * 2.0 +
                      2.0 * L.conv.kh * L.conv.kw * L.conv.cin * L.conv.cout;
            L.kind = L_STEMPOOL;
            L.sub = 2;
            L.klass = prof_class(h, conv_stempool_name());
            L.d_argv = g.d_args + first_blk[i] * slot;
            g.launches.push_back(L);
            continue;
        }
        if (chain[i] == 3) {                                     // a layer of a dense block: G blocks of each of its two convolutions
            double flop = 0, bytes = 0;
            for (int sub = 1; sub >= 0; sub--)
                for (int k = G - 1; k >= 0; k--) {
                    const Member& mk = h->members[h->workers[g.workers[k]].member];
                    const int rc = fill_args(h, h->workers[g.workers[k]], leader, G, mk.ops[i + sub], L);
                    if (rc != ENS_OK) return rc;
                    L.conv.ws = nullptr;
                    L.conv.ws_floats = 0;
                    if (k == 0) {
                        flop += L.flop;
                        if (sub == 1) {                          // algorithmic bytes: the block's input and weights, the appended channels
                            L.conv2 = L.conv;
                            bytes += (double)leader.batch * L.conv.H * L.conv.W * L.conv.cout * 2.0 + 2.0 * 9 * L.conv.cin * L.conv.cout;
                        } else {
                            bytes += (double)leader.batch * L.conv.H * L.conv.W * L.conv.cin * 2.0 + 2.0 * L.conv.cin * L.conv.cout;
                        }
                    }
                    memcpy(host.data() + (first_blk[i] + (size_t)sub * G + k) * slot, &L.conv, sizeof(ConvArgs));
                }
            L.kind = L_DENSE;
            L.sub = 2;
            L.flop = flop;
            L.bytes = bytes;
            L.klass = prof_class(h, conv_dense_name());
            L.d_argv = g.d_args + first_blk[i] * slot;
            g.launches.push_back(L);
            continue;
        }
        if (chain[i] == 1) {                                     // G blocks of each of the three convolutions
            double flop = 0, wbytes = 0;
            for (int sub = 2; sub >= 0; sub--)
                for (int k = G - 1; k >= 0; k--) {
                    const Member& mk = h->members[h->workers[g.workers[k]].member];
                    const int rc = fill_args(h, h->workers[g.workers[k]], leader, G, mk.ops[i + sub], L);
                    if (rc != ENS_OK) return rc;
                    L.conv.ws = nullptr;
                    L.conv.ws_floats = 0;
                    if (k == 0) {
                        flop += L.flop;
                        wbytes += 2.0 * L.conv.kh * L.conv.kw * L.conv.cin * L.conv.cout;
                        if (sub == 2) L.conv3 = L.conv;
                        if (sub == 1) L.conv2 = L.conv;
                    }
                    memcpy(host.data() + (first_blk[i] + (size_t)sub * G + k) * slot, &L.conv, sizeof(ConvArgs));
                }
            // algorithmic bytes of the block: input once (it is the residual too, unless that is another tensor), output, weights
            const double px = (double)leader.batch * L.conv.H * L.conv.W;
            const bool own_res = L.conv3.res.p && L.conv3.res.p != L.conv.x.p;
            L.kind = L_BNECK;
            L.sub = 3;
            L.flop = flop;
            L.bytes = px * 2.0 * (L.conv.cin + L.conv3.cout * (own_res ? 2 : 1)) + wbytes;
            L.klass = prof_class(h, conv_bneck_name(L.conv));
            L.d_argv = g.d_args + first_blk[i] * slot;
            g.launches.push_back(L);
            continue;
        }
        const int nsub = fused[i] == 1 ? 2 : (m.ops[i].sub > 1 ? m.ops[i].sub : 1);
        // the one with more output channels leads (the grid is sized for the first argument block), the
        // deeper of two equals (so is the tile shape)
        const bool second_leads = fused[i] == 1 &&
            (m.ops[i + 1].sub_cout > m.ops[i].sub_cout ||
             (m.ops[i + 1].sub_cout == m.ops[i].sub_cout &&
              m.ops[i + 1].op.kh * m.ops[i + 1].op.kw * m.ops[i + 1].cin_s > m.ops[i].op.kh * m.ops[i].op.kw * m.ops[i].cin_s));
        double flop2 = 0, bytes2 = 0;
        for (int sub = nsub - 1; sub >= 0; sub--)
            for (int k = G - 1; k >= 0; k--) {                   // (k, sub) == (0, 0) last: L keeps the leader's first block
                const Member& mk = h->members[h->workers[g.workers[k]].member];
                const OpPlan& pl = swapped[i] == 1 || swapped[i] == 3 ? mk.ops[i + 1] : swapped[i] == 2 || swapped[i] == 4 ? mk.ops[i - 1]
                                   : fused[i] == 1 && (sub == 1) != second_leads ? mk.ops[i + 1] : mk.ops[i];
                const int rc = fill_args(h, h->workers[g.workers[k]], leader, G, pl, L, fused[i] == 1 ? 0 : sub);
                if (rc != ENS_OK) return rc;
                if (swapped[i] >= 3) {
                    // the pool first: pre-activation and average of the convolution's input into the convolution's output
                    // memory, as many channels wide as that input; then the convolution over the pooled map, nothing in front
                    const Worker& wk = h->workers[g.workers[k]];
                    const OpPlan& c = swapped[i] == 3 ? mk.ops[i] : mk.ops[i - 1];
                    const OpPlan& q = swapped[i] == 3 ? mk.ops[i + 1] : mk.ops[i];
                    const TensorInfo &tx = mk.tensors[c.op.src], &tq = mk.tensors[q.op.dst];
                    View mid;
                    mid.p = wk.arena + wk.layout.offset[c.op.dst];
                    mid.stride = c.op.cin;
                    mid.c0 = 0;
                    const char* P = mk.dev_params;
                    if (swapped[i] == 3) {
                        L.pool.x = view_of(wk, leader, mk, c.op.src, c.op.src_c0);
                        L.pool.y = mid;
                        L.pool.c = c.op.cin;
                        L.pool.H = tx.h; L.pool.W = tx.w;
                        L.pool.pre_scale = (const float*)(P + c.pre_scale);
                        L.pool.pre_shift = (const float*)(P + c.pre_shift);
                        L.bytes = (double)wk.batch * ((double)tx.h * tx.w + (double)tq.h * tq.w) * c.op.cin * 2.0;
                        L.klass = prof_class(h, "window_kernel<avgpool,pre>");
                    } else {
                        L.conv.x = mid;
                        L.conv.y = view_of(wk, leader, mk, q.op.dst, q.op.dst_c0);
                        L.conv.pre_scale = L.conv.pre_shift = nullptr;
                        L.conv.H = L.conv.Ho = tq.h; L.conv.W = L.conv.Wo = tq.w;
                        L.conv.inv_hw = 1.0 / ((double)tq.h * tq.w); L.conv.inv_w = 1.0 / (double)tq.w;
                        L.flop = 2.0 * wk.batch * tq.h * tq.w * (double)c.op.cout * c.op.cin;
                        L.bytes = (double)wk.batch * tq.h * tq.w * (c.op.cin + c.op.cout) * 2.0 + (double)c.op.cin * c.op.cout * 2.0;
                        L.klass = prof_class(h, conv_bf16_variant_name(L.conv, G));
                    }
                } else if (swapped[i]) {
                    // the convolution first: from the pool's input into the pool's output memory, as many channels wide
                    // as the convolution has, batch-norm but no activation; then the pool over that, with the activation
                    const Worker& wk = h->workers[g.workers[k]];
                    const OpPlan& q = swapped[i] == 1 ? mk.ops[i] : mk.ops[i - 1];
                    const OpPlan& c = swapped[i] == 1 ? mk.ops[i + 1] : mk.ops[i];
                    View mid;
                    mid.p = wk.arena + wk.layout.offset[q.op.dst];
                    mid.stride = c.op.cout;
                    mid.c0 = 0;
                    const double px = (double)wk.batch * mk.tensors[q.op.dst].h * mk.tensors[q.op.dst].w;
                    if (swapped[i] == 1) {
                        L.conv.x = view_of(wk, leader, mk, q.op.src, q.op.src_c0);
                        L.conv.y = mid;
                        L.conv.act = ACT_NONE;
                        L.klass = prof_class(h, conv_bf16_variant_name(L.conv, G));
                    } else {
                        L.pool.x = mid;
                        L.pool.y = view_of(wk, leader, mk, c.op.dst, c.op.dst_c0);
                        L.pool.c = c.op.cout;
                        L.pool.act = c.op.act;
                        L.bytes = px * c.op.cout * 2.0 * 2.0;
                        L.klass = prof_class(h, "window_kernel<avgpool,act>");
                    }
                }
                const double se_pass = L.bytes / 3.0;            // squeeze-excite: the tensor is read twice and written once
                if (summed[i] == 1) {                            // the sums go to the scratch of the block behind
                    const Worker& wk = h->workers[g.workers[k]];
                    const OpPlan& se = mk.ops[i + 1];
                    L.pool.sums = (float*)(wk.arena + wk.layout.offset[se.scratch]);
                    L.pool.sums_stride = se_scratch_floats(se.op.cin, se.op.r, se.se_cap);
                    L.klass = prof_class(h, "window_kernel<dwconv,sums>");
                } else if (summed[i] == 2) {                     // one pass over the input less
                    L.se.have_sums = dwconv_sums_blocks(mk.tensors[pl.op.src].h, mk.tensors[pl.op.src].w, pl.op.cin);
                    L.bytes -= se_pass;
                }
                if (gated[i] == 1) {                             // the block stops at the gates: one pass over its input
                    L.se.gate_only = 1;
                    L.bytes -= 2.0 * se_pass;
                    if (summed[i] == 2) L.bytes = (double)L.se.nb * L.se.have_sums * L.se.c * sizeof(float);   // only the rows of sums
                } else if (gated[i] == 2) {
                    gate_args(h->workers[g.workers[k]], mk.ops[i - 1], L.conv);
                    L.klass = prof_class(h, conv_bf16_variant_name(L.conv, G));
                }
                if (fused[i] == 1) {                             // no split of the depth: the two would share one workspace
                    L.conv.wpk = nullptr;                        // the generic kernel runs both
                    L.conv.ws = nullptr;
                    L.conv.ws_floats = 0;
                    if (sub == 1) { flop2 = L.flop; bytes2 = L.bytes; }
                }
                char* dst = host.data() + (first_blk[i] + (size_t)sub * G + k) * slot;
                switch (L.kind) {
                    case L_CONV: memcpy(dst, &L.conv, sizeof(ConvArgs)); break;
                    case L_DWCONV:
                    case L_POOL: memcpy(dst, &L.pool, sizeof(PoolArgs)); break;
                    case L_GAP: memcpy(dst, &L.gap, sizeof(GapArgs)); break;
                    case L_FC: memcpy(dst, &L.fc, sizeof(FcArgs)); break;
                    case L_SE: memcpy(dst, &L.se, sizeof(SeArgs)); break;
                    default: break;
                }
            }
        if (fused[i] == 1) {
            L.sub = 2;
            L.flop += flop2;
            L.bytes += bytes2;
            L.klass = prof_class(h, conv_bf16_variant_name(L.conv, 2 * G));
        }
        L.d_argv = g.d_args + first_blk[i] * slot;
        g.launches.push_back(L);
    }
    // The device arrays are indexed by element size, so every block is re-packed densely.
    for (size_t i = 0; i < m.ops.size(); i++) {
        const Launch& L = g.launches[i];
        size_t sz = 0;
        switch (L.kind) {
            case L_CONV:
            case L_BNECK:
            case L_DENSE:
            case L_STEMPOOL: sz = sizeof(ConvArgs); break;
            case L_DWCONV:
            case L_POOL: sz = sizeof(PoolArgs); break;
            case L_GAP: sz = sizeof(GapArgs); break;
            case L_FC: sz = sizeof(FcArgs); break;
            case L_SE: sz = sizeof(SeArgs); break;
            default: break;
        }
        char* base = host.data() + first_blk[i] * slot;
        const size_t nb_i = first_blk[i + 1] - first_blk[i];
        for (size_t k = 1; k < nb_i; k++) memmove(base + k * sz, base + k * slot, sz);
    }
    g.stage.src = nullptr;                                       // bound per request
    g.stage.dst = leader.arena + leader.layout.offset[0];
    g.stage.nb = leader.batch; g.stage.sh = h->base_h; g.stage.sw = h->base_w;
    g.stage.dh = m.in_h; g.stage.dw = m.in_w; g.stage.dc = m.tensors[0].cs; g.stage.s2d = m.stem_s2d ? 1 : 0;
    g.d_stage = (const StageArgs*)(g.d_args + n_blk * slot);
    HIP_TRY(hipMemcpy(g.d_args, host.data(), host.size(), hipMemcpyHostToDevice));
    return ENS_OK;
}

static int ensure_buffers(ens_handle* h, int64_t n);

static void destroy_workers(ens_handle* h) {
    for (Gang& g : h->gangs) {
        if (g.stream) (void)hipStreamSynchronize(g.stream);
        if (g.d_args) (void)hipFree(g.d_args);
        if (g.done) (void)hipEventDestroy(g.done);
        if (g.stream) (void)hipStreamDestroy(g.stream);
    }
    h->gangs.clear();
    for (Worker& w : h->workers)
        if (w.arena) (void)hipFree(w.arena);
    h->workers.clear();
    h->have_alloc = false;
}

static int64_t alloc_bytes(const ens_handle* h, const ens_alloc& a) {
    int64_t total = 0;
    for (const Member& m : h->members) total += (int64_t)m.weight_bytes();
    for (int r = 0; r < a.rows; r++)
        for (int c = 0; c < a.cols; c++)
            if (a.batch[r][c] > 0) total += (int64_t)plan_arena(h->members[c], a.batch[r][c], h->keep_tensors).bytes;
    return total;
}

// The worker streams of an allocation run at once: each launch counts on its share of the chip.
static int stream_share(const ens_handle* h) {
    const int streams = (int)std::max<size_t>(1, h->gangs.size());
    return std::max(32, 256 / streams);
}

static int install_alloc(ens_handle* h, const ens_alloc& a, int segment_size) {
    const int M = (int)h->members.size();
    if (a.rows <= 0 || a.rows > ENS_MAX_SLOTS || a.cols != M) return ENS_E_INVALID;
    int max_batch = 0;
    for (int c = 0; c < M; c++) {
        bool any = false;
        for (int r = 0; r < a.rows; r++) {
            if (a.batch[r][c] < 0) return ENS_E_INVALID;
            any = any || a.batch[r][c] > 0;
            max_batch = std::max(max_batch, a.batch[r][c]);
        }
        if (!any) return ENS_E_INVALID;                          // a column of zeros is illegal
    }
    if (segment_size <= 0) segment_size = 128;
    segment_size = std::max(segment_size, max_batch);           // segment >= the largest batch size
    const int64_t need = alloc_bytes(h, a);
    if (h->budget && (uint64_t)need > h->budget) return ENS_E_NOMEM;
    destroy_workers(h);
    for (int r = 0; r < a.rows; r++)
        for (int c = 0; c < M; c++) {
            if (a.batch[r][c] == 0) continue;
            Worker w;
            w.member = c; w.batch = a.batch[r][c]; w.slot = r;
            w.layout = plan_arena(h->members[c], w.batch, h->keep_tensors);
            w.arena_bytes = w.layout.bytes;
            h->workers.push_back(w);
        }
    for (Worker& w : h->workers) {                               // rank among the member's workers
        w.rank = 0; w.of = 0;
        for (const Worker& u : h->workers)
            if (u.member == w.member) { if (u.slot < w.slot) w.rank++; w.of++; }
    }
    for (Worker& w : h->workers) {
        hipError_t e = hipMalloc((void**)&w.arena, std::max<size_t>(w.arena_bytes, 256));
        if (e != hipSuccess) {
            (void)hipGetLastError();
            destroy_workers(h);
            return e == hipErrorOutOfMemory ? ENS_E_NOMEM : ENS_E_HIP;
        }
    }
    // gangs: same row, same network shape and the same column of the matrix (hence the same batch size
    // here, the same fellow workers and so the same share of the segments)
    auto same_column = [&](int c1, int c2) {
        for (int r = 0; r < a.rows; r++)
            if (a.batch[r][c1] != a.batch[r][c2]) return false;
        return true;
    };
    for (size_t i = 0; i < h->workers.size(); i++) {
        Worker& w = h->workers[i];
        for (size_t gi = 0; gi < h->gangs.size() && w.gang < 0 && h->gangs_enabled; gi++) {
            const Worker& l = h->workers[h->gangs[gi].workers[0]];
            if (l.slot == w.slot && same_column(l.member, w.member) && same_network(h->members[l.member], h->members[w.member])) {
                w.gang = (int)gi;
                h->gangs[gi].workers.push_back((int)i);
            }
        }
        if (w.gang < 0) {
            Gang g;
            g.workers.push_back((int)i);
            g.rank = w.rank; g.of = w.of;
            w.gang = (int)h->gangs.size();
            h->gangs.push_back(g);
        }
    }
    if (!h->d_logits.empty() && !h->d_logits[0]) {               // argument blocks hold the logits pointers
        const int rc0 = ensure_buffers(h, 1);
        if (rc0 != ENS_OK) { destroy_workers(h); return rc0; }
    }
    cu_budget() = stream_share(h);
    for (Gang& g : h->gangs) {
        hipError_t e = hipStreamCreateWithFlags(&g.stream, hipStreamNonBlocking);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&g.done, hipEventDisableTiming);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            destroy_workers(h);
            return ENS_E_HIP;
        }
        const int rc = build_launches(h, g);
        if (rc != ENS_OK) { destroy_workers(h); return rc; }
    }
    h->args_stale = false;
    h->bound_images = nullptr;
    h->alloc = a;
    h->alloc.bytes = need;
    h->segment_size = segment_size;
    h->have_alloc = true;
    return ENS_OK;
}

static hipEvent_t take_event(ens_handle* h) {
    if (!h->event_pool.empty()) {
        hipEvent_t e = h->event_pool.back();
        h->event_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

static hipError_t issue(const Launch& L, bool bf16, int G, int nb, long long first, hipStream_t s) {
    switch (L.kind) {
        case L_CONV: return bf16 ? launch_conv_bf16(L.conv, (const ConvArgs*)L.d_argv, G * L.sub, nb, s)
                                 : launch_conv_f32(L.conv, (const ConvArgs*)L.d_argv, G * L.sub, nb, s);
        case L_DWCONV: return launch_dwconv(L.pool, (const PoolArgs*)L.d_argv, G, nb, bf16, s);
        case L_POOL: return launch_pool(L.pool, (const PoolArgs*)L.d_argv, G, nb, L.is_max, bf16, s);
        case L_GAP: return launch_gap(L.gap, (const GapArgs*)L.d_argv, G, nb, bf16, s);
        case L_FC: return launch_fc(L.fc, (const FcArgs*)L.d_argv, G, nb, first, bf16, s);
        case L_SE: return launch_se(L.se, (const SeArgs*)L.d_argv, G, nb, bf16, s);
        case L_BNECK: return launch_conv_bneck(L.conv, L.conv2, L.conv3, (const ConvArgs*)L.d_argv, G, nb, s);
        case L_DENSE: return launch_conv_dense(L.conv, L.conv2, (const ConvArgs*)L.d_argv, G, nb, s);
        case L_STEMPOOL: return launch_conv_stempool(L.conv, L.conv2, (const ConvArgs*)L.d_argv, G, nb, s);
        case L_SKIP: return hipSuccess;
    }
    return hipErrorInvalidValue;
}

// One batch of one gang: stage the images into the leader's arena, run every member, write the
// logits rows of the batch.
static int forward_batch(ens_handle* h, Gang& g, int64_t first, int nb) {
    const hipStream_t st = h->one_stream ? h->main_stream : g.stream;
    const Worker& leader = h->workers[g.workers[0]];
    const Member& m = h->members[leader.member];
    const int G = (int)g.workers.size();
    const double scale = (double)nb / leader.batch;
    auto timed = [&](int klass, double flop, double bytes, auto&& fn) -> hipError_t {
        if (!h->profiling) return fn();
        ProfRec r{klass, take_event(h), take_event(h), flop * scale, bytes * scale};
        if (!r.start || !r.stop) return hipErrorOutOfMemory;
        next_launch_events() = LaunchEvents{r.start, r.stop};    // stamped with the kernels' own begin and end
        const hipError_t e = fn();
        next_launch_events() = LaunchEvents{};
        h->prof_recs.push_back(r);
        return e;
    };
    if (h->fake_predictor) {                                     // zeros for the rows of this batch, nothing else
        for (int wi : g.workers) {
            const Worker& w = h->workers[wi];
            HIP_TRY(launch_fill_zero(h->d_logits[w.member] + first * h->classes, (int64_t)nb * h->classes, st));
            h->workers[wi].last_nb = nb;
        }
        return ENS_OK;
    }
    const double stage_bytes = (double)leader.batch * (h->base_h * h->base_w * 12.0 + (double)m.tensors[0].h * m.tensors[0].w * g.stage.dc * (m.bf16 ? 2 : 4));
    HIP_TRY(timed(h->stage_klass, 0.0, stage_bytes, [&] { return launch_stage(g.stage, g.d_stage, 1, nb, first, m.bf16, st); }));
    for (const Launch& L : g.launches) {
        if (L.kind == L_SKIP) continue;
        HIP_TRY(timed(L.klass, L.flop * G, L.bytes * G, [&] { return issue(L, m.bf16, G, nb, first, st); }));
    }
    for (int wi : g.workers) h->workers[wi].last_nb = nb;
    return ENS_OK;
}

static int ensure_buffers(ens_handle* h, int64_t n) {
    const size_t rows = (size_t)n;
    bool moved = false;
    if (rows > h->d_logits_heap_rows) {
        for (float*& p : h->d_logits_heap) {
            if (p) (void)hipFree(p);
            p = nullptr;
        }
        h->d_logits_heap.assign(h->members.size(), nullptr);
        h->d_logits_heap_rows = 0;
        for (size_t m = 0; m < h->members.size(); m++)
            HIP_TRY(hipMalloc((void**)&h->d_logits_heap[m], rows * h->members[m].classes * sizeof(float)));
        h->d_logits_heap_rows = rows;
        if (!h->d_logit_ptrs) HIP_TRY(hipMalloc((void**)&h->d_logit_ptrs, ENS_MAX_MEMBERS * sizeof(float*)));
        moved = true;
    }
    if (moved || h->logits_static || h->d_logit_table != h->d_logit_ptrs) {   // (back) to the library's own buffers
        h->d_logits = h->d_logits_heap;
        h->d_logits_rows = h->d_logits_heap_rows;
        h->d_logit_table = h->d_logit_ptrs;
        h->logits_static = false;
        h->args_stale = true;                                  // the FC argument blocks name these buffers
        HIP_TRY(hipMemcpy((void*)h->d_logit_ptrs, h->d_logits.data(), h->members.size() * sizeof(float*), hipMemcpyHostToDevice));
    }
    return ENS_OK;
}

// Points the per-member logits at slices of the fixed device array: a table of the members' pointers
// in its first bytes, then one block of `rows` x classes floats per member.  Allocates nothing.
static int use_static_logits(ens_handle* h, int64_t n) {
    void* base = nullptr;
    size_t bytes = 0;
    HIP_TRY(static_scratch(&base, &bytes));
    const size_t M = h->members.size();
    const size_t row_bytes = M * (size_t)h->classes * sizeof(float);
    const size_t rows_cap = (bytes - STATIC_SCRATCH_TABLE_BYTES) / row_bytes;
    if ((size_t)n > rows_cap) {
        fprintf(stderr, "ens_predict_static: %lld images x %zu members x %d classes of fp32 logits exceed the %zu-byte "
                "static scratch (at most %zu images for this ensemble)\n", (long long)n, M, h->classes, bytes, rows_cap);
        return ENS_E_TOOBIG;
    }
    float* first = (float*)((char*)base + STATIC_SCRATCH_TABLE_BYTES);
    const bool there = h->logits_static && h->d_logit_table == (const float**)base && !h->d_logits.empty() && h->d_logits[0] == first;
    if (!there) {
        h->d_logits.assign(M, nullptr);
        for (size_t m = 0; m < M; m++) h->d_logits[m] = first + m * rows_cap * (size_t)h->classes;
        h->d_logits_rows = rows_cap;
        h->d_logit_table = (const float**)base;
        h->logits_static = true;
        h->args_stale = true;                                  // the FC argument blocks name these buffers
    }
    // the table is written on every call: another handle's call may have left its own there
    HIP_TRY(hipMemcpy(base, h->d_logits.data(), M * sizeof(float*), hipMemcpyHostToDevice));
    return ENS_OK;
}

static int grow(float** p, size_t* cap, size_t want_floats) {
    if (want_floats <= *cap) return ENS_OK;
    if (*p) (void)hipFree(*p);
    *p = nullptr;
    *cap = 0;
    HIP_TRY(hipMalloc((void**)p, want_floats * sizeof(float)));
    *cap = want_floats;
    return ENS_OK;
}

// f(X, A) -> Y with X and Y on the device.  `mask` selects the members that take part (all
// members for a real request; a single member when the BBS baseline times it alone).
// may_alloc false (the allocation-free entry point): the logits buffers are already in place and
// nothing on the way may allocate or free device memory.
static int run_device(ens_handle* h, const float* d_images, int64_t n, float* d_probs, uint64_t mask, bool may_alloc = true) {
    if (n == 0) return ENS_OK;
    cu_budget() = stream_share(h);
    int rc = may_alloc ? ensure_buffers(h, n) : ENS_OK;
    if (rc != ENS_OK) return rc;
    if ((size_t)n > h->d_logits_rows) return ENS_E_INVALID;
    const int M = (int)h->members.size();
    const int seg = h->segment_size;
    const int64_t n_seg = (n + seg - 1) / seg;
    if (h->args_stale || h->bound_images != d_images) {          // (re)bind request buffers in the argument blocks
        for (Gang& g : h->gangs) {
            if (h->args_stale) {
                rc = build_launches(h, g, may_alloc);
                if (rc != ENS_OK) return rc;
            }
            g.stage.src = d_images;
            g.stage.sh = h->base_h; g.stage.sw = h->base_w;
            HIP_TRY(hipMemcpyAsync((void*)g.d_stage, &g.stage, sizeof(StageArgs), hipMemcpyHostToDevice, h->main_stream));
        }
        h->args_stale = false;
        h->bound_images = d_images;
    }
    // the workers start once the request images are in place on the main stream
    HIP_TRY(hipEventRecord(h->input_ready, h->main_stream));
    for (Gang& g : h->gangs) HIP_TRY(hipStreamWaitEvent(g.stream, h->input_ready, 0));
    // every segment id goes once to every member; a member's workers share its segments as they
    // would by taking them from one queue, the faster worker more of them (planner.cpp, hand_out)
    std::vector<std::vector<int32_t>> owner(M);
    for (int c = 0; c < M; c++) {
        std::vector<int32_t> batches;
        const Gang* first = nullptr;
        for (const Worker& w : h->workers)                       // in slot order = rank order
            if (w.member == c) {
                batches.push_back(w.batch);
                if (w.rank == 0) first = &h->gangs[w.gang];
            }
        if (batches.size() <= 1 || !first) continue;
        double flop = 0;
        int launches = 1;
        for (const Launch& L : first->launches)
            if (L.kind != L_SKIP) { flop += L.flop; launches++; }
        const double launch_cost = launches * 8e-6;              // a kernel of a small batch lasts about this long whatever it does
        const double image_cost = flop / batches[0] / (h->members[c].bf16 ? 4e14 : 2e13);
        rc = hand_out(n, seg, batches.data(), (int)batches.size(), launch_cost, image_cost, &owner[c]);
        if (rc != ENS_OK) return rc;
    }
    for (int64_t s = 0; s < n_seg; s++) {
        const int64_t start = s * seg, end = std::min<int64_t>((s + 1) * seg, n);
        for (Gang& g : h->gangs) {
            const int member0 = h->workers[g.workers[0]].member;
            if (g.of > 1 && owner[member0][s] != g.rank) continue;
            bool wanted = false;
            for (int wi : g.workers) wanted = wanted || ((mask >> h->workers[wi].member) & 1);
            if (!wanted) continue;
            const int b = h->workers[g.workers[0]].batch;
            for (int64_t a = start; a < end; a += b) {
                rc = forward_batch(h, g, a, (int)std::min<int64_t>(b, end - a));
                if (rc != ENS_OK) return rc;
            }
        }
    }
    for (Gang& g : h->gangs) {
        HIP_TRY(hipEventRecord(g.done, g.stream));
        HIP_TRY(hipStreamWaitEvent(h->main_stream, g.done, 0));
    }
    if (mask == ~0ull || M == 1) {
        ProfRec r{prof_class(h, "combine_kernel"), nullptr, nullptr, 0.0, (double)n * h->classes * 4.0 * (M + 1)};
        if (h->profiling) {
            r.start = take_event(h); r.stop = take_event(h);
            if (!r.start || !r.stop) return ENS_E_HIP;
            next_launch_events() = LaunchEvents{r.start, r.stop};
        }
        HIP_TRY(launch_combine(h->d_logit_table, h->d_weights, h->combine_rule, M, n, h->classes, d_probs, h->main_stream));
        if (h->profiling) {
            next_launch_events() = LaunchEvents{};
            h->prof_recs.push_back(r);
        }
    }
    return ENS_OK;
}

static int finish_profile(ens_handle* h) {
    for (ProfRec& r : h->prof_recs) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            ProfClass& c = h->prof[r.klass];
            c.ms += ms; c.flop += r.flop; c.bytes += r.bytes; c.launches++;
        }
        h->event_pool.push_back(r.start);
        h->event_pool.push_back(r.stop);
    }
    h->prof_recs.clear();
    return ENS_OK;
}

static void reset_profile(ens_handle* h) {
    for (ProfClass& c : h->prof) { c.ms = 0; c.flop = 0; c.bytes = 0; c.launches = 0; }
}

static int default_alloc(ens_handle* h) {
    ens_alloc a;
    memset(&a, 0, sizeof(a));
    a.rows = 1;
    a.cols = (int)h->members.size();
    for (int c = 0; c < a.cols; c++) a.batch[0][c] = 8;
    return install_alloc(h, a, 128);
}

static int ensure_calib(ens_handle* h, int64_t n) {
    if ((size_t)n <= h->d_calib_images) return ENS_OK;
    if (h->d_calib) (void)hipFree(h->d_calib);
    h->d_calib = nullptr;
    h->d_calib_images = 0;
    const size_t count = (size_t)n * h->base_h * h->base_w * 3;
    HIP_TRY(hipMalloc((void**)&h->d_calib, count * sizeof(float)));
    HIP_TRY(launch_fill_noise(h->d_calib, (int64_t)count, 0x5EEDCA11Bull, h->main_stream));
    HIP_TRY(hipStreamSynchronize(h->main_stream));
    h->d_calib_images = (size_t)n;
    return ENS_OK;
}

// Benchmark Mode on the installed allocation: median images/s of `repeats` runs after a warm-up.
static int time_installed(ens_handle* h, int64_t n, int repeats, uint64_t mask, double* ips) {
    int rc = ensure_calib(h, n);
    if (rc != ENS_OK) return rc;
    rc = grow(&h->d_probs, &h->d_probs_cap, (size_t)n * h->classes);
    if (rc != ENS_OK) return rc;
    std::vector<double> secs;
    for (int i = 0; i < repeats + 1; i++) {
        const auto t0 = std::chrono::steady_clock::now();
        rc = run_device(h, h->d_calib, n, h->d_probs, mask);
        if (rc != ENS_OK) return rc;
        HIP_TRY(hipStreamSynchronize(h->main_stream));
        const auto t1 = std::chrono::steady_clock::now();
        if (i > 0) secs.push_back(std::chrono::duration<double>(t1 - t0).count());
    }
    if (h->profiling) finish_profile(h);
    std::sort(secs.begin(), secs.end());
    *ips = (double)n / secs[secs.size() / 2];
    return ENS_OK;
}

}  // namespace ens

// ------------------------------------------------------------------------------------ C API
extern "C" {

int ens_load(const ens_member_spec* specs, int32_t n_members, uint64_t seed, ens_handle** out) {
    if (!specs || !out || n_members <= 0 || n_members > ENS_MAX_MEMBERS) return ENS_E_INVALID;
    *out = nullptr;
    ens_handle* h = new ens_handle();
    memset(&h->alloc, 0, sizeof(h->alloc));
    for (int i = 0; i < n_members; i++) {
        const ens_member_spec& sp = specs[i];
        std::vector<float> drawn;
        const float* params = sp.params;
        if (!params) {
            if (!sp.param_specs || sp.n_params <= 0) { delete h; return ENS_E_INVALID; }
            drawn.assign((size_t)sp.n_params, 0.f);
            const int rc = draw_params(sp.param_specs, sp.n_param_specs, seed, i, drawn.data(), sp.n_params);
            if (rc != ENS_OK) { delete h; return rc; }
            params = drawn.data();
        }
        Member m;
        const int rc = build_member(sp, params, &m);
        if (rc != ENS_OK) { delete h; return rc; }
        h->members.push_back(std::move(m));
    }
    h->classes = h->members[0].classes;
    for (const Member& m : h->members)
        if (m.classes != h->classes) { delete h; return ENS_E_INVALID; }
    h->base_h = h->members[0].in_h;
    h->base_w = h->members[0].in_w;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        delete h;
        return ENS_E_NODEVICE;
    }
    auto fail = [&](int rc) { ens_free(h); return rc; };
    for (Member& m : h->members) {
        hipError_t e = hipMalloc((void**)&m.dev_params, std::max<size_t>(m.host_params.size(), 256));
        if (e == hipSuccess)
            e = hipMemcpy(m.dev_params, m.host_params.data(), m.host_params.size(), hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return fail(e == hipErrorOutOfMemory ? ENS_E_NOMEM : ENS_E_HIP);
        }
    }
    if (hipStreamCreateWithFlags(&h->main_stream, hipStreamNonBlocking) != hipSuccess) return fail(ENS_E_HIP);
    if (hipEventCreateWithFlags(&h->input_ready, hipEventDisableTiming) != hipSuccess) return fail(ENS_E_HIP);
    h->d_logits.assign(h->members.size(), nullptr);
    h->stage_klass = prof_class(h, "stage_kernel");
    *out = h;
    return ENS_OK;
}

void ens_free(ens_handle* h) {
    if (!h) return;
    (void)hipDeviceSynchronize();
    destroy_workers(h);
    for (Member& m : h->members)
        if (m.dev_params) (void)hipFree(m.dev_params);
    for (float* p : h->d_logits_heap)
        if (p) (void)hipFree(p);
    if (h->d_logit_ptrs) (void)hipFree((void*)h->d_logit_ptrs);
    if (h->d_weights) (void)hipFree(h->d_weights);
    if (h->d_images) (void)hipFree(h->d_images);
    if (h->d_probs) (void)hipFree(h->d_probs);
    if (h->d_calib) (void)hipFree(h->d_calib);
    for (ProfRec& r : h->prof_recs) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    for (hipEvent_t e : h->event_pool) (void)hipEventDestroy(e);
    if (h->input_ready) (void)hipEventDestroy(h->input_ready);
    if (h->main_stream) (void)hipStreamDestroy(h->main_stream);
    delete h;
}

int ens_set_io(ens_handle* h, int32_t base_h, int32_t base_w, int32_t images_on_device, int32_t probs_on_device) {
    if (!h || base_h <= 0 || base_w <= 0) return ENS_E_INVALID;
    if (base_h != h->base_h || base_w != h->base_w) {
        if (h->d_calib) (void)hipFree(h->d_calib);
        h->d_calib = nullptr;
        h->d_calib_images = 0;
    }
    h->base_h = base_h;
    h->base_w = base_w;
    h->bound_images = nullptr;
    h->images_on_device = images_on_device != 0;
    h->probs_on_device = probs_on_device != 0;
    return ENS_OK;
}

int ens_set_alloc(ens_handle* h, const ens_alloc* a, int32_t segment_size) {
    if (!h || !a) return ENS_E_INVALID;
    return install_alloc(h, *a, segment_size);
}

int ens_predict(ens_handle* h, const float* images, int64_t n, float* probs_out) {
    if (!h || n < 0 || (n > 0 && (!images || !probs_out))) return ENS_E_INVALID;
    if (n == 0) return ENS_OK;
    if (!h->have_alloc) {
        const int rc = default_alloc(h);
        if (rc != ENS_OK) return rc;
    }
    const auto t0 = std::chrono::steady_clock::now();
    const size_t img_floats = (size_t)n * h->base_h * h->base_w * 3;
    const float* d_in = images;
    if (!h->images_on_device) {
        int rc = grow(&h->d_images, &h->d_images_cap, img_floats);
        if (rc != ENS_OK) return rc;
        HIP_TRY(hipMemcpyAsync(h->d_images, images, img_floats * sizeof(float), hipMemcpyHostToDevice, h->main_stream));
        d_in = h->d_images;
    }
    float* d_out = probs_out;
    if (!h->probs_on_device) {
        int rc = grow(&h->d_probs, &h->d_probs_cap, (size_t)n * h->classes);
        if (rc != ENS_OK) return rc;
        d_out = h->d_probs;
    }
    if (h->profiling) reset_profile(h);
    int rc = run_device(h, d_in, n, d_out, ~0ull);
    if (rc != ENS_OK) { (void)hipDeviceSynchronize(); return rc; }
    if (!h->probs_on_device)
        HIP_TRY(hipMemcpyAsync(probs_out, d_out, (size_t)n * h->classes * sizeof(float), hipMemcpyDeviceToHost, h->main_stream));
    HIP_TRY(hipStreamSynchronize(h->main_stream));
    if (h->profiling) finish_profile(h);
    h->last_n = n;
    h->last_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    return ENS_OK;
}

int ens_predict_static(ens_handle* h, const float* d_images, int64_t n, float* d_probs_out) {
    if (!h || n < 0 || (n > 0 && (!d_images || !d_probs_out))) return ENS_E_INVALID;
    if (!h->have_alloc || h->profiling) {
        fprintf(stderr, "ens_predict_static: %s\n", !h->have_alloc ? "no allocation installed (ens_plan or ens_set_alloc first)"
                                                                   : "per-kernel profiling creates events: switch it off");
        return ENS_E_INVALID;
    }
    if (n == 0) return ENS_OK;
    const auto t0 = std::chrono::steady_clock::now();
    int rc = use_static_logits(h, n);
    if (rc != ENS_OK) return rc;
    rc = run_device(h, d_images, n, d_probs_out, ~0ull, false);
    if (rc != ENS_OK) { (void)hipDeviceSynchronize(); return rc; }
    HIP_TRY(hipStreamSynchronize(h->main_stream));
    h->last_n = n;
    h->last_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    return ENS_OK;
}

int ens_static_scratch_bytes(void) { return (int)STATIC_SCRATCH_BYTES; }

int ens_bench(ens_handle* h, const ens_alloc* a, int32_t segment_size, int64_t n_calib, int32_t repeats,
              double* img_per_sec) {
    if (!h || !a || !img_per_sec || n_calib <= 0) return ENS_E_INVALID;
    if (repeats <= 0) repeats = 3;
    *img_per_sec = 0.0;
    int rc = install_alloc(h, *a, segment_size);
    if (rc == ENS_E_NOMEM) return ENS_OK;                        // a matrix that does not fit scores zero (Algorithm 2, definition of bench)
    if (rc != ENS_OK) return rc;
    if (h->profiling) reset_profile(h);
    return time_installed(h, n_calib, repeats, ~0ull, img_per_sec);
}

int ens_plan(ens_handle* h, uint64_t mem_budget_bytes, const ens_plan_opts* opts, ens_alloc* out) {
    if (!h || !out) return ENS_E_INVALID;
    ens_plan_opts o;
    memset(&o, 0, sizeof(o));
    if (opts) o = *opts;
    if (o.n_domain <= 0) {
        const int d[5] = {8, 16, 32, 64, 128};
        o.n_domain = 5;
        memcpy(o.domain, d, sizeof(d));
    }
    if (o.n_domain > ENS_MAX_DOMAIN) return ENS_E_INVALID;
    if (o.default_batch <= 0) o.default_batch = *std::min_element(o.domain, o.domain + o.n_domain);
    if (o.segment_size <= 0) o.segment_size = 128;
    if (o.max_neighs <= 0) o.max_neighs = 100;
    if (o.max_iter <= 0) o.max_iter = 10;
    if (o.slots <= 0) o.slots = 1;
    if (o.slots > ENS_MAX_SLOTS) return ENS_E_INVALID;
    if (o.n_calib <= 0) o.n_calib = 1024;
    if (o.repeats <= 0) o.repeats = 3;
    const int M = (int)h->members.size();
    if (mem_budget_bytes == 0) {
        size_t fr = 0, tot = 0;
        HIP_TRY(hipMemGetInfo(&fr, &tot));
        mem_budget_bytes = tot;
    }
    h->budget = mem_budget_bytes;

    std::vector<int64_t> wbytes(M), abytes((size_t)M * o.n_domain);
    for (int m = 0; m < M; m++) {
        wbytes[m] = (int64_t)h->members[m].weight_bytes();
        for (int j = 0; j < o.n_domain; j++) abytes[(size_t)m * o.n_domain + j] = (int64_t)plan_arena(h->members[m], o.domain[j]).bytes;
    }
    std::vector<int32_t> row_pool(o.slots, 0), row_gpu(o.slots, 1);
    // request buffers (images, logits, probabilities) come out of the same budget
    int64_t reserve = (int64_t)o.n_calib * ((int64_t)h->base_h * h->base_w * 3 + (int64_t)h->classes * (M + 1)) * 4;
    int64_t cap = (int64_t)mem_budget_bytes - reserve;
    if (cap < 0) cap = 0;
    ens_plan_problem p;
    p.n_models = M; p.n_rows = o.slots; p.n_pools = 1; p.n_domain = o.n_domain;
    p.domain = o.domain; p.default_batch = o.default_batch;
    p.weight_bytes = wbytes.data(); p.arena_bytes = abytes.data();
    p.row_pool = row_pool.data(); p.row_is_gpu = row_gpu.data(); p.pool_cap = &cap;
    p.max_iter = o.max_iter; p.max_neighs = o.max_neighs; p.seed = o.seed;
    if (!problem_ok(&p)) return ENS_E_INVALID;

    std::vector<int32_t> A((size_t)o.slots * M, 0);
    int rc = wfd(p, A.data());
    if (rc != ENS_OK) return rc;
    auto to_alloc = [&](const int32_t* mat) {
        ens_alloc a;
        memset(&a, 0, sizeof(a));
        a.rows = o.slots; a.cols = M;
        for (int r = 0; r < o.slots; r++)
            for (int c = 0; c < M; c++) a.batch[r][c] = mat[r * M + c];
        return a;
    };
    int hip_rc = ENS_OK;
    int32_t shown = 0;
    auto show = [&](const int32_t* mat, double ips) {             // progress of a long plan
        if (!o.verbose) return;
        std::string line;
        for (int r = 0; r < o.slots; r++) {
            line += r ? " | " : "";
            for (int c = 0; c < M; c++) line += (c ? " " : "") + std::to_string(mat[r * M + c]);
        }
        fprintf(stderr, "ens_plan: benchmark %d: [%s] -> %.1f images/s\n", ++shown, line.c_str(), ips);
        fflush(stderr);
    };
    auto bench = [&](const int32_t* mat) -> double {
        if (!fit_mem(p, mat)) return 0.0;
        const ens_alloc a = to_alloc(mat);
        double ips = 0.0;
        const int r = ens_bench(h, &a, o.segment_size, o.n_calib, o.repeats, &ips);
        if (r != ENS_OK) { hip_rc = r; return 0.0; }
        show(mat, ips);
        return ips;
    };
    double score = 0.0;
    int32_t n_bench = 0;
    if (o.strategy == 0) {
        rc = greedy(p, A.data(), bench, &score, &n_bench);
    } else if (o.strategy == 1) {
        score = bench(A.data());
        n_bench = 1;
    } else if (o.strategy == 2) {
        // each member alone on the GPU, its batch size scanned; then the combined matrix is timed
        std::vector<int32_t> best(M, o.default_batch);
        auto single = [&](int m, int b) -> double {
            std::vector<int32_t> mat((size_t)o.slots * M, 0);
            for (int c = 0; c < M; c++) mat[c] = c == m ? b : o.default_batch;
            if (!fit_mem(p, mat.data())) return 0.0;
            const ens_alloc a = to_alloc(mat.data());
            h->gangs_enabled = false;                            // the member is timed alone
            int r = install_alloc(h, a, o.segment_size);
            h->gangs_enabled = true;
            if (r == ENS_E_NOMEM) return 0.0;
            if (r != ENS_OK) { hip_rc = r; return 0.0; }
            double ips = 0.0;
            r = time_installed(h, o.n_calib, o.repeats, 1ull << m, &ips);
            if (r != ENS_OK) { hip_rc = r; return 0.0; }
            show(mat.data(), ips);
            return ips;
        };
        rc = bbs(p, single, best.data(), &n_bench);
        std::fill(A.begin(), A.end(), 0);
        for (int c = 0; c < M; c++) A[c] = best[c];
        score = bench(A.data());
    } else {
        return ENS_E_INVALID;
    }
    if (rc != ENS_OK) return rc;
    if (hip_rc != ENS_OK) return hip_rc;
    ens_alloc a = to_alloc(A.data());
    rc = install_alloc(h, a, o.segment_size);
    if (rc != ENS_OK) return rc;
    *out = h->alloc;
    out->score = score;
    out->n_bench = n_bench;
    h->alloc = *out;
    return ENS_OK;
}

int ens_member_logits(ens_handle* h, int32_t member, int64_t n, float* logits_out) {
    if (!h || member < 0 || member >= (int)h->members.size() || !logits_out) return ENS_E_INVALID;
    if (n <= 0 || n > h->last_n || (size_t)n > h->d_logits_rows) return ENS_E_INVALID;
    HIP_TRY(hipMemcpy(logits_out, h->d_logits[member], (size_t)n * h->members[member].classes * sizeof(float),
                      hipMemcpyDeviceToHost));
    return ENS_OK;
}

int ens_debug_tensor(ens_handle* h, int32_t member, int32_t tensor, int32_t n_images, float* out) {
    if (!h || !out || member < 0 || member >= (int)h->members.size()) return ENS_E_INVALID;
    const Member& m = h->members[member];
    if (tensor < 0 || tensor >= (int)m.tensors.size() || m.tensors[tensor].external) return ENS_E_INVALID;
    const Worker* w = nullptr;
    for (const Worker& x : h->workers)
        if (x.member == member) { w = &x; break; }
    if (!w || n_images <= 0 || n_images > w->last_nb) return ENS_E_INVALID;
    if (tensor == 0) w = &h->workers[h->gangs[w->gang].workers[0]];   // the staged input lives with the gang's leader
    const TensorInfo& ti = m.tensors[tensor];
    const size_t elems = (size_t)n_images * ti.elems_per_image();
    std::vector<uint8_t> raw(elems * (ti.f32 ? 4 : 2));
    HIP_TRY(hipMemcpy(raw.data(), w->arena + w->layout.offset[tensor], raw.size(), hipMemcpyDeviceToHost));
    const size_t pixels = (size_t)n_images * ti.h * ti.w;
    for (size_t p = 0; p < pixels; p++)
        for (int c = 0; c < ti.c; c++) {
            float v;
            if (ti.f32) {
                v = ((const float*)raw.data())[p * ti.cs + c];
            } else {
                const uint32_t u = ((uint32_t)((const uint16_t*)raw.data())[p * ti.cs + c]) << 16;
                memcpy(&v, &u, 4);
            }
            out[p * ti.c + c] = v;
        }
    return ENS_OK;
}

int ens_debug_keep_tensors(ens_handle* h, int32_t on) {
    if (!h) return ENS_E_INVALID;
    h->keep_tensors = on != 0;
    return ENS_OK;
}

int ens_classes(const ens_handle* h) { return h ? h->classes : ENS_E_INVALID; }
int ens_n_members(const ens_handle* h) { return h ? (int)h->members.size() : ENS_E_INVALID; }

int ens_member_bytes(const ens_handle* h, int32_t member, int32_t batch, int64_t* weight_bytes, int64_t* arena_bytes) {
    if (!h || member < 0 || member >= (int)h->members.size() || batch <= 0) return ENS_E_INVALID;
    if (weight_bytes) *weight_bytes = (int64_t)h->members[member].weight_bytes();
    if (arena_bytes) *arena_bytes = (int64_t)plan_arena(h->members[member], batch).bytes;
    return ENS_OK;
}

int ens_spec_bytes(const ens_member_spec* spec, int32_t batch, int64_t* weight_bytes, int64_t* arena_bytes) {
    if (!spec || batch <= 0) return ENS_E_INVALID;
    std::vector<float> zeros;
    const float* params = spec->params;
    if (!params) {
        if (spec->n_params <= 0) return ENS_E_INVALID;
        zeros.assign((size_t)spec->n_params, 0.f);
        params = zeros.data();
    }
    Member m;
    const int rc = build_member(*spec, params, &m);
    if (rc != ENS_OK) return rc;
    if (weight_bytes) *weight_bytes = (int64_t)m.weight_bytes();
    if (arena_bytes) *arena_bytes = (int64_t)plan_arena(m, batch).bytes;
    return ENS_OK;
}

int ens_debug_fake_predictor(ens_handle* h, int32_t on) {
    if (!h) return ENS_E_INVALID;
    h->fake_predictor = on != 0;
    return ENS_OK;
}

int ens_set_combination(ens_handle* h, int32_t rule, const float* weights) {
    if (!h) return ENS_E_INVALID;
    if (rule != ENS_COMBINE_MEAN && rule != ENS_COMBINE_WEIGHTED && rule != ENS_COMBINE_VOTE) return ENS_E_INVALID;
    if (rule == ENS_COMBINE_WEIGHTED) {
        if (!weights) return ENS_E_INVALID;
        if (!h->d_weights) HIP_TRY(hipMalloc((void**)&h->d_weights, ENS_MAX_MEMBERS * sizeof(float)));
        HIP_TRY(hipMemcpy(h->d_weights, weights, h->members.size() * sizeof(float), hipMemcpyHostToDevice));
    }
    h->combine_rule = rule;
    return ENS_OK;
}

int ens_debug_one_stream(ens_handle* h, int32_t on) {
    if (!h) return ENS_E_INVALID;
    (void)hipDeviceSynchronize();
    h->one_stream = on != 0;
    return ENS_OK;
}

int ens_set_profiling(ens_handle* h, int32_t on) {
    if (!h) return ENS_E_INVALID;
    h->profiling = on != 0;
    return ENS_OK;
}

int ens_profile_get(const ens_handle* h, int32_t idx, char* name, int32_t name_len, double* ms, int64_t* launches,
                    double* flop, double* bytes) {
    if (!h || idx < 0 || idx >= (int)h->prof.size()) return ENS_E_INVALID;
    const ProfClass& c = h->prof[idx];
    if (name && name_len > 0) {
        strncpy(name, c.name.c_str(), (size_t)name_len - 1);
        name[name_len - 1] = 0;
    }
    if (ms) *ms = c.ms;
    if (launches) *launches = c.launches;
    if (flop) *flop = c.flop;
    if (bytes) *bytes = c.bytes;
    return ENS_OK;
}

double ens_last_ms(const ens_handle* h) { return h ? h->last_ms : 0.0; }

const char* ens_strerror(int status) {
    switch (status) {
        case ENS_OK: return "ok";
        case ENS_E_INVALID: return "invalid description, matrix or argument";
        case ENS_E_NOMEM: return "not enough device memory for a member or worker";
        case ENS_E_NOFIT: return "no device has enough memory for a member";
        case ENS_E_HIP: return "HIP runtime error";
        case ENS_E_NODEVICE: return "no GPU visible";
        case ENS_E_UNSUPPORTED: return "shape not covered by the GPU kernels";
        case ENS_E_TOOBIG: return "request larger than the static scratch of the allocation-free entry point";
    }
    return "unknown status";
}

const char* ens_version(void) { return "ens-mi355x 0.1 (gfx950)"; }

}  // extern "C"
