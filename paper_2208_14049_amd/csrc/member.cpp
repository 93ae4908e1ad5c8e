// Host-side preparation of a member: validation of its description, batch-norm folding,
// conversion of the parameters to the device layout, and liveness-based placement of its
// activation tensors in a worker's arena.  No GPU calls in this file.
#include <algorithm>
#include <cmath>
#include <cstring>

#include "engine.h"

namespace ens {

static const double BN_EPS = 1e-5;
static const size_t ALIGN = 256;

static uint16_t to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

struct BlobWriter {
    std::vector<uint8_t>& buf;
    size_t reserve(size_t bytes) {
        const size_t off = align_up(buf.size());
        buf.resize(off + bytes, 0);
        return off;
    }
    size_t put_f32(const std::vector<float>& v) {
        const size_t off = reserve(v.size() * 4);
        memcpy(buf.data() + off, v.data(), v.size() * 4);
        return off;
    }
    size_t put(const std::vector<float>& v, bool bf16) {
        if (!bf16) return put_f32(v);
        const size_t off = reserve(v.size() * 2);
        uint16_t* d = (uint16_t*)(buf.data() + off);
        for (size_t i = 0; i < v.size(); i++) d[i] = to_bf16(v[i]);
        return off;
    }
};

static bool in_blob(int64_t off, int64_t n, int64_t total) { return off >= 0 && n >= 0 && off + n <= total; }

// scale[c] = gamma / sqrt(var + eps), shift[c] = beta - mean * scale
static void bn_affine(const float* bn, int C, std::vector<float>* scale, std::vector<float>* shift) {
    scale->resize(C);
    shift->resize(C);
    for (int c = 0; c < C; c++) {
        const double s = (double)bn[c] / std::sqrt((double)bn[3 * C + c] + BN_EPS);
        (*scale)[c] = (float)s;
        (*shift)[c] = (float)((double)bn[C + c] - (double)bn[2 * C + c] * s);
    }
}

int build_member(const ens_member_spec& spec, const float* params, Member* out) {
    if (!spec.tensors || !spec.ops || spec.n_tensors <= 0 || spec.n_ops <= 0 || !params) return ENS_E_INVALID;
    if (spec.out_tensor <= 0 || spec.out_tensor >= spec.n_tensors) return ENS_E_INVALID;
    if (spec.dtype != ENS_FP32 && spec.dtype != ENS_BF16) return ENS_E_INVALID;
    Member m;
    m.bf16 = spec.dtype == ENS_BF16;
    const int NT = spec.n_tensors;
    const int64_t NP = spec.n_params;
    if (spec.tensors[0].c != 3) return ENS_E_UNSUPPORTED;       // requests are 3-channel images
    m.in_h = spec.tensors[0].h;
    m.in_w = spec.tensors[0].w;
    m.out_tensor = spec.out_tensor;
    m.classes = spec.tensors[spec.out_tensor].c;
    if (spec.tensors[spec.out_tensor].h != 1 || spec.tensors[spec.out_tensor].w != 1) return ENS_E_INVALID;

    m.tensors.resize(NT);
    for (int t = 0; t < NT; t++) {
        const ens_tensor& s = spec.tensors[t];
        if (s.h <= 0 || s.w <= 0 || s.c <= 0) return ENS_E_INVALID;
        TensorInfo& ti = m.tensors[t];
        ti.h = s.h; ti.w = s.w; ti.c = s.c;
        ti.cs = s.c;
        ti.f32 = !m.bf16;
        ti.def = t == 0 ? -1 : INT32_MAX;
        ti.last = -1;
        ti.external = false;
    }
    // outputs of the global pool and the FC head are fp32 vectors whatever the member's dtype
    for (int i = 0; i < spec.n_ops; i++) {
        const ens_op& o = spec.ops[i];
        if (o.dst <= 0 || o.dst >= NT || o.src < 0 || o.src >= NT) return ENS_E_INVALID;
        if (o.kind == ENS_OP_GAP || o.kind == ENS_OP_FC) m.tensors[o.dst].f32 = true;
    }
    if (m.bf16)
        for (int t = 0; t < NT; t++)
            if (!m.tensors[t].f32) m.tensors[t].cs = (m.tensors[t].c + 7) / 8 * 8;

    // A stride-2 convolution that is the only reader of the 3-channel input image is run as a
    // stride-1 convolution over the image stored space-to-depth: with image row 2r + b in channel
    // group b of row r, filter row k at padding p becomes filter row floor((k - p) / 2) of group
    // (k - p) mod 2.  A 7x7 filter turns into 4x4 taps of 12 channels, stored 16 wide: K drops
    // from 49 x 8 to 16 x 16 and every tap is a 32-byte run instead of 16 bytes.
    int stem_op = -1;
    if (m.bf16) {
        int readers = 0;
        for (int i = 0; i < spec.n_ops; i++) {
            const ens_op& o = spec.ops[i];
            if (o.src == 0) { readers++; stem_op = i; }
            if (o.kind == ENS_OP_CONV && o.res == 0) readers += 2;
        }
        if (readers != 1) stem_op = -1;
        if (stem_op >= 0) {
            const ens_op& o = spec.ops[stem_op];
            if (o.kind != ENS_OP_CONV || o.sh != 2 || o.sw != 2 || o.cin != 3 || o.src_c0 != 0 || o.pre ||
                o.kh < 2 || o.kw < 2 || o.kh > 8 || o.kw > 8)
                stem_op = -1;
        }
    }

    BlobWriter bw{m.host_params};
    m.zeros_off = bw.reserve(256);
    bool seen_out = false;
    for (int i = 0; i < spec.n_ops; i++) {
        const ens_op& o = spec.ops[i];
        OpPlan pl;
        pl.op = o;
        pl.w = pl.b = pl.scale = pl.pre_scale = pl.pre_shift = pl.w2 = pl.b2 = pl.w_packed = SIZE_MAX;
        pl.cin_s = o.cin;
        pl.scratch = -1;
        pl.alg_k = 0;
        pl.sub = 1;
        pl.sub_cout = o.cout;
        pl.fuse_next = false;
        pl.fuse_chain = false;
        pl.fuse_dense = false;
        pl.fuse_pool = false;
        pl.fuse_gate = false;
        pl.fuse_sums = false;
        pl.swap_pool = false;
        pl.swap_conv = false;
        pl.se_cap = SE_MAX_SPLITS;
        TensorInfo& ts = m.tensors[o.src];
        TensorInfo& td = m.tensors[o.dst];
        if (o.cin <= 0 || o.cout <= 0 || o.src_c0 < 0 || o.dst_c0 < 0) return ENS_E_INVALID;
        if (o.src_c0 + o.cin > ts.c || o.dst_c0 + o.cout > td.c) return ENS_E_INVALID;
        if (ts.def == INT32_MAX) return ENS_E_INVALID;           // read before written
        if (o.dst == spec.out_tensor) {
            if (o.kind != ENS_OP_FC || seen_out) return ENS_E_UNSUPPORTED;
            seen_out = true;
        }
        ts.last = std::max(ts.last, i);
        td.def = std::min(td.def, i);
        td.last = std::max(td.last, i);
        // Two convolutions in a row over the same input slice with same-sized outputs may run as one launch:
        // the second output is then written while the first operation runs.
        if (m.bf16 && i > 0 && o.kind == ENS_OP_CONV && spec.ops[i - 1].kind == ENS_OP_CONV) {
            const ens_op& q = spec.ops[i - 1];
            const TensorInfo& tq = m.tensors[q.dst];
            if (q.src == o.src && q.src_c0 == o.src_c0 && q.cin == o.cin && q.sh == o.sh && q.sw == o.sw &&
                tq.h == td.h && tq.w == td.w && o.src != q.dst && o.res != q.dst && o.src != 0 &&
                (q.dst != o.dst || q.dst_c0 + q.cout <= o.dst_c0 || o.dst_c0 + o.cout <= q.dst_c0) &&   // disjoint outputs
                q.r <= 1 && o.r <= 1 && !q.pre && !o.pre && !m.ops[i - 1].fuse_next && (i < 2 || !m.ops[i - 2].fuse_next)) {
                m.ops[i - 1].fuse_next = true;
                td.def = std::min(td.def, i - 1);
            }
        }
        const bool windowed = o.kind == ENS_OP_CONV || o.kind == ENS_OP_DWCONV || o.kind == ENS_OP_MAXPOOL ||
                              o.kind == ENS_OP_AVGPOOL;
        if (windowed) {
            if (o.kh <= 0 || o.kw <= 0 || o.sh <= 0 || o.sw <= 0 || o.pt < 0 || o.pl < 0) return ENS_E_INVALID;
            if (ts.f32 != !m.bf16 || td.f32 != !m.bf16) return ENS_E_UNSUPPORTED;
            // every output pixel must have its window origin inside the padded input
            if ((td.h - 1) * o.sh - o.pt >= ts.h || (td.w - 1) * o.sw - o.pl >= ts.w) return ENS_E_INVALID;
        }
        // 16-byte channel granularity of the bf16 kernels
        auto aligned8 = [&](int c0, int c) { return c0 % 8 == 0 && c % 8 == 0; };
        switch (o.kind) {
            case ENS_OP_CONV: {
                // r > 1: that many groups; output channel co sees the input channels of group co / (cout / r)
                const int groups = o.r > 1 ? o.r : 1;
                if (o.cin % groups || o.cout % groups) return ENS_E_INVALID;
                const int ig = o.cin / groups, og = o.cout / groups;
                // groups per dense sub-convolution: as many as make 32 output channels (the matrix-core
                // block), the whole group when it is wider than that
                const int per_sub = og >= 32 ? 1 : 32 / og;
                if (groups > 1) {
                    if (!m.bf16 || o.pre || (og < 32 && 32 % og) || groups % per_sub) return ENS_E_UNSUPPORTED;
                    if ((per_sub * ig) % 8 || (per_sub * og) % 8) return ENS_E_UNSUPPORTED;
                }
                const int64_t nw = (int64_t)o.kh * o.kw * ig * o.cout;
                if (!in_blob(o.off_w, nw, NP)) return ENS_E_INVALID;
                if (o.off_b >= 0 && !in_blob(o.off_b, o.cout, NP)) return ENS_E_INVALID;
                if (o.off_bn >= 0 && !in_blob(o.off_bn, 4 * (int64_t)o.cout, NP)) return ENS_E_INVALID;
                if (o.pre && !in_blob(o.off_pre, 4 * (int64_t)o.cin, NP)) return ENS_E_INVALID;
                if (m.bf16) {
                    if (o.src == 0 && ts.c % 8) {               // the padded input image
                        if (o.src_c0 != 0 || o.cin != ts.c) return ENS_E_UNSUPPORTED;
                        pl.cin_s = ts.cs;
                    } else if (!aligned8(o.src_c0, o.cin)) {
                        return ENS_E_UNSUPPORTED;
                    }
                    if (!aligned8(o.dst_c0, o.cout)) return ENS_E_UNSUPPORTED;
                }
                if (o.res >= 0) {
                    if (o.res >= NT || o.res_c0 < 0 || o.res_c0 + o.cout > m.tensors[o.res].c) return ENS_E_INVALID;
                    TensorInfo& tr = m.tensors[o.res];
                    if (tr.h != td.h || tr.w != td.w || tr.def == INT32_MAX) return ENS_E_INVALID;
                    if (m.bf16 && o.res_c0 % 8) return ENS_E_UNSUPPORTED;
                    tr.last = std::max(tr.last, i);
                }
                std::vector<float> scale(o.cout, 1.f), shift(o.cout, 0.f);
                if (o.off_bn >= 0) bn_affine(params + o.off_bn, o.cout, &scale, &shift);
                // bf16 members: the weights stay as given and the kernels multiply the fp32 sum by the scale;
                // fp32 members: the scale goes into the weights (wscale) and the kernels see ones
                std::vector<float> wscale(o.cout, 1.f);
                if (!m.bf16) { wscale = scale; }
                const float* w = params + o.off_w;               // [kh][kw][cin][cout]
                std::vector<float> wf;
                if (i == stem_op) {
                    auto floor2 = [](int v) { return v >= 0 ? v / 2 : -((1 - v) / 2); };
                    const int ah0 = floor2(-o.pt), ah1 = floor2(o.kh - 1 - o.pt);
                    const int aw0 = floor2(-o.pl), aw1 = floor2(o.kw - 1 - o.pl);
                    const int kh2 = ah1 - ah0 + 1, kw2 = aw1 - aw0 + 1;
                    wf.assign((size_t)o.cout * kh2 * kw2 * 16, 0.f);
                    for (int co = 0; co < o.cout; co++)
                        for (int kh = 0; kh < o.kh; kh++)
                            for (int kw = 0; kw < o.kw; kw++) {
                                const int ah = floor2(kh - o.pt), bh = kh - o.pt - 2 * ah;
                                const int aw = floor2(kw - o.pl), bw2 = kw - o.pl - 2 * aw;
                                for (int ci = 0; ci < 3; ci++)
                                    wf[(((size_t)co * kh2 + (ah - ah0)) * kw2 + (aw - aw0)) * 16 + (bh * 2 + bw2) * 3 + ci] =
                                        w[((size_t)(kh * o.kw + kw) * 3 + ci) * o.cout + co] * wscale[co];
                            }
                    pl.alg_k = o.kh * o.kw * o.cin;
                    pl.op.kh = kh2; pl.op.kw = kw2; pl.op.sh = 1; pl.op.sw = 1;
                    pl.op.pt = -ah0; pl.op.pl = -aw0; pl.op.cin = 12;
                    pl.cin_s = 16;
                } else if (groups > 1) {
                    // [sub][sub_cout][kh*kw][cin_s]: dense blocks of per_sub groups, zeros between groups
                    pl.sub = groups / per_sub;
                    pl.sub_cout = per_sub * og;
                    pl.cin_s = per_sub * ig;
                    wf.assign((size_t)o.cout * o.kh * o.kw * pl.cin_s, 0.f);
                    for (int co = 0; co < o.cout; co++) {
                        const int g = co / og;
                        const int ci0 = (g % per_sub) * ig;     // the group's place among its block's input channels
                        for (int k = 0; k < o.kh * o.kw; k++)
                            for (int ci = 0; ci < ig; ci++)
                                wf[((size_t)co * o.kh * o.kw + k) * pl.cin_s + ci0 + ci] =
                                    w[((size_t)k * ig + ci) * o.cout + co] * wscale[co];
                    }
                } else {
                    wf.assign((size_t)o.cout * o.kh * o.kw * pl.cin_s, 0.f);
                    for (int co = 0; co < o.cout; co++)
                        for (int k = 0; k < o.kh * o.kw; k++)
                            for (int ci = 0; ci < o.cin; ci++)
                                wf[((size_t)co * o.kh * o.kw + k) * pl.cin_s + ci] =
                                    w[((size_t)k * o.cin + ci) * o.cout + co] * wscale[co];
                }
                std::vector<float> bias(o.cout);
                for (int co = 0; co < o.cout; co++)
                    bias[co] = (o.off_b >= 0 ? params[o.off_b + co] * scale[co] : 0.f) + shift[co];
                pl.w = bw.put(wf, m.bf16);
                pl.b = bw.put_f32(bias);
                pl.scale = bw.put_f32(m.bf16 ? scale : std::vector<float>(o.cout, 1.f));
                if (o.pre) {
                    std::vector<float> ps, ph;
                    bn_affine(params + o.off_pre, o.cin, &ps, &ph);
                    ps.resize(pl.cin_s, 0.f);
                    ph.resize(pl.cin_s, 0.f);
                    pl.pre_scale = bw.put_f32(ps);
                    pl.pre_shift = bw.put_f32(ph);
                }
                break;
            }
            case ENS_OP_DWCONV: {
                if (o.cin != o.cout) return ENS_E_INVALID;
                const int64_t nw = (int64_t)o.kh * o.kw * o.cin;
                if (!in_blob(o.off_w, nw, NP)) return ENS_E_INVALID;
                if (o.off_b >= 0 && !in_blob(o.off_b, o.cout, NP)) return ENS_E_INVALID;
                if (o.off_bn >= 0 && !in_blob(o.off_bn, 4 * (int64_t)o.cout, NP)) return ENS_E_INVALID;
                if (m.bf16 && (!aligned8(o.src_c0, o.cin) || o.dst_c0 % 8)) return ENS_E_UNSUPPORTED;
                if (o.pre || o.res >= 0) return ENS_E_UNSUPPORTED;
                std::vector<float> scale(o.cout, 1.f), shift(o.cout, 0.f);
                if (o.off_bn >= 0) bn_affine(params + o.off_bn, o.cout, &scale, &shift);
                std::vector<float> wf((size_t)nw), bias(o.cout);
                for (int k = 0; k < o.kh * o.kw; k++)
                    for (int c = 0; c < o.cin; c++) wf[(size_t)k * o.cin + c] = params[o.off_w + (size_t)k * o.cin + c] * (m.bf16 ? 1.f : scale[c]);
                for (int c = 0; c < o.cout; c++)
                    bias[c] = (o.off_b >= 0 ? params[o.off_b + c] * scale[c] : 0.f) + shift[c];
                pl.w = bw.put(wf, m.bf16);
                pl.b = bw.put_f32(bias);
                pl.scale = bw.put_f32(m.bf16 ? scale : std::vector<float>(o.cout, 1.f));
                break;
            }
            case ENS_OP_MAXPOOL:
            case ENS_OP_AVGPOOL:
                if (o.cin != o.cout) return ENS_E_INVALID;
                if (m.bf16 && (!aligned8(o.src_c0, o.cin) || o.dst_c0 % 8)) return ENS_E_UNSUPPORTED;
                break;
            case ENS_OP_GAP: {
                if (o.cin != o.cout || td.h != 1 || td.w != 1) return ENS_E_INVALID;
                if (ts.f32 != !m.bf16) return ENS_E_UNSUPPORTED;
                if (o.pre) {
                    if (!in_blob(o.off_pre, 4 * (int64_t)o.cin, NP)) return ENS_E_INVALID;
                    std::vector<float> ps, ph;
                    bn_affine(params + o.off_pre, o.cin, &ps, &ph);
                    pl.pre_scale = bw.put_f32(ps);
                    pl.pre_shift = bw.put_f32(ph);
                }
                break;
            }
            case ENS_OP_FC: {
                if (ts.h != 1 || ts.w != 1 || td.h != 1 || td.w != 1 || !ts.f32) return ENS_E_UNSUPPORTED;
                if (o.src_c0 != 0 || o.cin != ts.c || o.dst_c0 != 0 || o.cout != td.c) return ENS_E_UNSUPPORTED;
                if (!in_blob(o.off_w, (int64_t)o.cin * o.cout, NP) || !in_blob(o.off_b, o.cout, NP)) return ENS_E_INVALID;
                std::vector<float> wf(params + o.off_w, params + o.off_w + (size_t)o.cin * o.cout);
                std::vector<float> bias(params + o.off_b, params + o.off_b + o.cout);
                pl.w = bw.put(wf, m.bf16);
                pl.b = bw.put_f32(bias);
                if (m.bf16 && o.cin % 8 == 0) {
                    // A second copy, transposed to [cout][cin] and in matrix-core operand order (see
                    // pack_operand_order below: blocks of 32 rows, steps of 16 columns, a lane's 8 values in a
                    // row), for the FC kernel that runs on the matrix cores.
                    const int rows = o.cout, K = o.cin;
                    const int rows_p = (rows + 31) / 32 * 32, K_p = (K + 63) / 64 * 64, NS = K_p / 16;
                    std::vector<float> wt((size_t)rows_p * K_p, 0.f);
                    for (int rb = 0; rb < rows_p / 32; rb++)
                        for (int st = 0; st < NS; st++)
                            for (int lane = 0; lane < 64; lane++) {
                                const int r = lane & 31, hh = lane >> 5;
                                const int row = 32 * rb + ((r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1)), col = 16 * st + 8 * hh;
                                if (row >= rows) continue;
                                for (int e = 0; e < 8 && col + e < K; e++)
                                    wt[(((size_t)rb * NS + st) * 64 + lane) * 8 + e] = wf[(size_t)(col + e) * o.cout + row];
                            }
                    pl.w_packed = bw.put(wt, true);
                }
                break;
            }
            case ENS_OP_SE: {
                if (o.cin != o.cout || o.r <= 0 || ts.h != td.h || ts.w != td.w) return ENS_E_INVALID;
                if (ts.f32 != !m.bf16 || td.f32 != !m.bf16) return ENS_E_UNSUPPORTED;
                if (m.bf16 && (!aligned8(o.src_c0, o.cin) || o.dst_c0 % 8)) return ENS_E_UNSUPPORTED;
                const int64_t n1 = (int64_t)o.cin * o.r;
                if (!in_blob(o.off_w, n1, NP) || !in_blob(o.off_b, o.r, NP) || !in_blob(o.off_w2, n1, NP) ||
                    !in_blob(o.off_b2, o.cin, NP))
                    return ENS_E_INVALID;
                pl.w = bw.put_f32(std::vector<float>(params + o.off_w, params + o.off_w + n1));
                pl.b = bw.put_f32(std::vector<float>(params + o.off_b, params + o.off_b + o.r));
                pl.w2 = bw.put_f32(std::vector<float>(params + o.off_w2, params + o.off_w2 + n1));
                pl.b2 = bw.put_f32(std::vector<float>(params + o.off_b2, params + o.off_b2 + o.cin));
                TensorInfo sc;                                   // per-image scratch: partial sums, hidden, gates
                sc.def = i;
                if (m.bf16 && i > 0) {                           // behind a depthwise convolution whose kernel can leave the sums
                    const ens_op& d = spec.ops[i - 1];
                    if (d.kind == ENS_OP_DWCONV && d.dst == o.src && d.dst_c0 == o.src_c0 && d.cin == o.cin && d.kh == d.kw &&
                        (d.kh == 3 || d.kh == 5) && d.sh == d.sw && (d.sh == 1 || d.sh == 2) && o.cin % 8 == 0) {
                        m.ops[i - 1].fuse_sums = true;
                        pl.se_cap = std::max((int)SE_MAX_SPLITS, dwconv_sums_blocks(ts.h, ts.w, o.cin));
                        sc.def = i - 1;
                    }
                }
                sc.h = 1; sc.w = 1; sc.c = sc.cs = se_scratch_floats(o.cin, o.r, pl.se_cap);
                sc.f32 = true; sc.last = i; sc.external = false;
                pl.scratch = (int)m.tensors.size();
                m.tensors.push_back(sc);
                break;
            }
            default:
                return ENS_E_INVALID;
        }
        m.ops.push_back(pl);
    }
    if (!seen_out) return ENS_E_INVALID;
    // Residual bottlenecks: 1x1, 3x3 (stride 1, padding 1), 1x1 in a row, each reading what the one
    // before wrote, with nobody else reading or writing the two tensors in between.  One kernel can
    // run all three (decided per batch size when the launches are built); the block's output then
    // counts as written from the first of them on.
    // Kernels that take each wavefront's weights straight from memory read a second copy of them in the
    // order of the matrix-core operands, so that a wavefront's load is 1 KB in a row.  Rows in blocks of
    // 32, the K axis (taps x channels) in steps of 16: [block][step][lane][8], lane (r, h) holding row
    // 32 block + r', columns 16 step + 8 h .. + 7, r' = r with bits 2 and 3 swapped.  Rows are padded with
    // zeros to a multiple of 32, columns to a multiple of 64.
    auto pack_operand_order = [&](OpPlan& pl) {
        if (pl.w_packed != SIZE_MAX) return;
        const int rows = pl.op.cout, K = pl.op.kh * pl.op.kw * pl.cin_s;       // K in 8s: a lane's 16 bytes are real or padding as a whole
        const int rows_p = (rows + 31) / 32 * 32, K_p = (K + 63) / 64 * 64;
        const size_t off = bw.reserve((size_t)rows_p * K_p * 2);
        const uint16_t* src = (const uint16_t*)(m.host_params.data() + pl.w);
        uint16_t* dst = (uint16_t*)(m.host_params.data() + off);
        const int NS = K_p / 16;
        for (int rb = 0; rb < rows_p / 32; rb++)
            for (int st = 0; st < NS; st++)
                for (int lane = 0; lane < 64; lane++) {
                    const int r = lane & 31, h = lane >> 5;
                    const int row = 32 * rb + ((r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1)), col = 16 * st + 8 * h;
                    if (row < rows && col < K) memcpy(dst + (((size_t)rb * NS + st) * 64 + lane) * 8, src + (size_t)row * K + col, 16);
                }
        pl.w_packed = off;
    };
    // 1x1 layers without padding or pre-activation (stride 1, or the strided shortcuts of residual stages): the kernel of conv_pw.hip
    if (m.bf16) {
        for (int i = 0; i < spec.n_ops; i++) {
            const ens_op& o = spec.ops[i];
            if (o.kind == ENS_OP_CONV && o.kh == 1 && o.kw == 1 && o.sh >= 1 && o.sw >= 1 && o.pt == 0 && o.pl == 0 && o.r <= 1 &&
                !o.pre && o.cin % 8 == 0 && o.cout % 8 == 0 && m.ops[i].cin_s == o.cin)
                pack_operand_order(m.ops[i]);
        }
    }
    if (m.bf16) {
        std::vector<int> uses(m.tensors.size(), 0);              // readers and writers of every tensor
        for (int i = 0; i < spec.n_ops; i++) {
            const ens_op& o = spec.ops[i];
            uses[o.src]++;
            uses[o.dst]++;
            if (o.kind == ENS_OP_CONV && o.res >= 0) uses[o.res]++;
        }
        auto plain = [](const ens_op& o, int k, int pad) {
            return o.kind == ENS_OP_CONV && o.kh == k && o.kw == k && o.sh == 1 && o.sw == 1 && o.pt == pad && o.pl == pad &&
                   o.r <= 1 && !o.pre;
        };
        for (int i = 0; i + 2 < spec.n_ops; i++) {
            const ens_op &p = spec.ops[i], &q = spec.ops[i + 1], &o = spec.ops[i + 2];
            if (!plain(p, 1, 0) || !plain(q, 3, 1) || !plain(o, 1, 0) || p.res >= 0 || q.res >= 0) continue;
            if (q.src != p.dst || q.src_c0 != p.dst_c0 || q.cin != p.cout || o.src != q.dst || o.src_c0 != q.dst_c0 || o.cin != q.cout) continue;
            if (p.cout != q.cout || (p.cout != 64 && p.cout != 128)) continue;
            if (uses[p.dst] != 2 || uses[q.dst] != 2 || p.dst == q.dst) continue;
            if (p.src == 0 || o.dst == p.src || o.dst == p.dst || o.dst == q.dst || o.res == p.dst || o.res == q.dst) continue;
            if (m.tensors[p.dst].c != p.cout || m.tensors[q.dst].c != q.cout) continue;      // whole tensors, not slices
            if (m.ops[i].fuse_next || m.ops[i + 1].fuse_next || m.ops[i + 2].fuse_next) continue;
            if (i > 1 && m.ops[i - 2].fuse_chain) continue;      // chains do not overlap
            if (i > 0 && m.ops[i - 1].fuse_chain) continue;
            if (p.cin % 32 || o.cout % 32) continue;
            m.ops[i].fuse_chain = true;
            m.tensors[o.dst].def = std::min(m.tensors[o.dst].def, i);
            for (int j = 0; j < 3; j++) pack_operand_order(m.ops[i + j]);
        }
    }
    // Layers of dense blocks: pre-activated 1x1 to 128 channels, then 3x3 (stride 1, padding 1) to 32 channels,
    // the tensor in between read by nobody else.  One kernel can run both (decided per batch size).
    if (m.bf16) {
        std::vector<int> uses(m.tensors.size(), 0);
        for (int i = 0; i < spec.n_ops; i++) {
            const ens_op& o = spec.ops[i];
            uses[o.src]++;
            uses[o.dst]++;
            if (o.kind == ENS_OP_CONV && o.res >= 0) uses[o.res]++;
        }
        for (int i = 0; i + 1 < spec.n_ops; i++) {
            const ens_op &p = spec.ops[i], &q = spec.ops[i + 1];
            if (p.kind != ENS_OP_CONV || q.kind != ENS_OP_CONV || !p.pre || q.pre || p.r > 1 || q.r > 1 || p.res >= 0 || q.res >= 0) continue;
            if (p.kh != 1 || p.kw != 1 || p.sh != 1 || p.sw != 1 || p.pt != 0 || p.pl != 0) continue;
            if (q.kh != 3 || q.kw != 3 || q.sh != 1 || q.sw != 1 || q.pt != 1 || q.pl != 1) continue;
            if (p.cout != 128 || q.cin != 128 || q.cout != 32 || p.cin % 32 || p.cin > 2048 || m.ops[i].cin_s != p.cin) continue;
            if (q.src != p.dst || q.src_c0 != p.dst_c0 || uses[p.dst] != 2 || m.tensors[p.dst].c != p.cout || p.src == 0) continue;
            if (q.dst == p.dst || (q.dst == p.src && q.dst_c0 < p.src_c0 + p.cin)) continue;
            if (m.ops[i].fuse_next || m.ops[i + 1].fuse_next || m.ops[i].fuse_chain || (i > 0 && m.ops[i - 1].fuse_chain) ||
                (i > 1 && m.ops[i - 2].fuse_chain) || m.ops[i + 1].fuse_chain)
                continue;
            m.ops[i].fuse_dense = true;
            // the one kernel writes the second output while it still reads the first input
            m.tensors[q.dst].def = std::min(m.tensors[q.dst].def, i);
            pack_operand_order(m.ops[i]);
            pack_operand_order(m.ops[i + 1]);
        }
    }
    // Squeeze-excite followed by a 1x1 convolution (stride 1, no pre-activation, not grouped) that alone reads its output
    if (m.bf16) {
        for (int i = 0; i + 1 < spec.n_ops; i++) {
            const ens_op &e = spec.ops[i], &c = spec.ops[i + 1];
            if (e.kind != ENS_OP_SE || c.kind != ENS_OP_CONV) continue;
            if (c.kh != 1 || c.kw != 1 || c.sh != 1 || c.sw != 1 || c.pt != 0 || c.pl != 0 || c.r > 1 || c.pre) continue;
            if (c.src != e.dst || c.src_c0 != e.dst_c0 || c.cin != e.cin || e.dst == e.src || c.dst == e.src || c.dst == e.dst) continue;
            if (m.ops[i + 1].w_packed == SIZE_MAX || m.ops[i + 1].fuse_next || m.ops[i + 1].fuse_chain || m.ops[i + 1].fuse_dense) continue;
            if (i > 0 && m.ops[i - 1].fuse_next) continue;
            int readers = 0;
            for (int k = 0; k < spec.n_ops; k++) {
                const ens_op& o = spec.ops[k];
                readers += o.src == e.dst;
                readers += o.kind == ENS_OP_CONV && o.res == e.dst;
            }
            if (readers != 1 || m.tensors[e.dst].c != e.cin || m.tensors[e.src].c < e.src_c0 + e.cin) continue;
            m.ops[i].fuse_gate = true;
            // the convolution then reads the block's input and its scratch (the gates)
            m.tensors[e.src].last = std::max(m.tensors[e.src].last, i + 1);
            m.tensors[m.ops[i].scratch].last = std::max(m.tensors[m.ops[i].scratch].last, i + 1);
        }
    }
    // A 3x3 / stride-1 / padding-1 average pool followed by a plain 1x1 convolution that alone reads its output
    if (m.bf16) {
        for (int i = 0; i + 1 < spec.n_ops; i++) {
            const ens_op &q = spec.ops[i], &c = spec.ops[i + 1];
            if (q.kind != ENS_OP_AVGPOOL || c.kind != ENS_OP_CONV) continue;
            if (q.kh != 3 || q.kw != 3 || q.sh != 1 || q.sw != 1 || q.pt != 1 || q.pl != 1) continue;
            if (c.kh != 1 || c.kw != 1 || c.sh != 1 || c.sw != 1 || c.pt != 0 || c.pl != 0 || c.r > 1 || c.pre || c.res >= 0) continue;
            if (c.src != q.dst || q.dst_c0 != 0 || c.src_c0 != 0 || c.cin != q.cin || m.tensors[q.dst].c != q.cin) continue;
            if (q.dst == q.src || c.dst == q.dst || c.cout > q.cin || c.cout % 8) continue;
            if (m.ops[i + 1].fuse_next || m.ops[i + 1].fuse_chain || m.ops[i + 1].fuse_dense || m.ops[i + 1].fuse_pool) continue;
            if (i > 0 && m.ops[i - 1].fuse_next) continue;
            int readers = 0;
            for (int k = 0; k < spec.n_ops; k++) {
                const ens_op& o = spec.ops[k];
                readers += o.src == q.dst;
                readers += o.kind == ENS_OP_CONV && o.res == q.dst;
            }
            if (readers != 1) continue;
            m.ops[i].swap_pool = true;
        }
    }
    // A pre-activated 1x1 convolution with no activation, followed by a 2x2 / stride-2 average pool that alone reads its output
    if (m.bf16) {
        for (int i = 0; i + 1 < spec.n_ops; i++) {
            const ens_op &c = spec.ops[i], &q = spec.ops[i + 1];
            if (c.kind != ENS_OP_CONV || q.kind != ENS_OP_AVGPOOL) continue;
            if (q.kh != 2 || q.kw != 2 || q.sh != 2 || q.sw != 2 || q.pt != 0 || q.pl != 0) continue;
            if (c.kh != 1 || c.kw != 1 || c.sh != 1 || c.sw != 1 || c.pt != 0 || c.pl != 0 || c.r > 1 || !c.pre || c.res >= 0 ||
                c.act != ENS_ACT_NONE)
                continue;
            if (q.src != c.dst || c.dst_c0 != 0 || q.src_c0 != 0 || q.cin != c.cout || m.tensors[c.dst].c != c.cout) continue;
            if (c.dst == c.src || q.dst == c.dst || c.cin % 8 || c.cout % 8 || m.ops[i].cin_s != c.cin) continue;
            if (m.ops[i].fuse_next || m.ops[i].fuse_chain || m.ops[i].fuse_dense || m.ops[i].fuse_pool) continue;
            if (i > 0 && (m.ops[i - 1].fuse_next || m.ops[i - 1].fuse_dense)) continue;
            const TensorInfo &tu = m.tensors[c.dst], &tq = m.tensors[q.dst];
            if ((long long)tq.h * tq.w * c.cin > (long long)tu.h * tu.w * c.cout) continue;   // the pooled input fits the middle tensor
            int readers = 0;
            for (int k = 0; k < spec.n_ops; k++) {
                const ens_op& o = spec.ops[k];
                readers += o.src == c.dst;
                readers += o.kind == ENS_OP_CONV && o.res == c.dst;
            }
            if (readers != 1) continue;
            m.ops[i].swap_conv = true;
            pack_operand_order(m.ops[i]);                        // behind the pool it is a plain 1x1 layer: the kernel of conv_pw.hip
        }
    }
    // The rewritten stem followed by a 3x3 / stride-2 / padding-1 max-pool that alone reads its output
    if (stem_op >= 0 && stem_op + 1 < spec.n_ops) {
        const ens_op &c = spec.ops[stem_op], &q = spec.ops[stem_op + 1];
        int readers = 0;
        for (int i = 0; i < spec.n_ops; i++) {
            const ens_op& o = spec.ops[i];
            readers += o.src == c.dst;
            readers += o.kind == ENS_OP_CONV && o.res == c.dst;
        }
        if (q.kind == ENS_OP_MAXPOOL && q.src == c.dst && q.src_c0 == c.dst_c0 && q.cin == c.cout && readers == 1 &&
            q.kh == 3 && q.kw == 3 && q.sh == 2 && q.sw == 2 && q.pt == 1 && q.pl == 1 && c.act == ENS_ACT_RELU && c.res < 0 &&
            m.tensors[c.dst].c == c.cout && q.dst != c.dst && q.dst != 0 && m.ops[stem_op].op.kh == 4 && m.ops[stem_op].op.kw == 4 &&
            !m.ops[stem_op].fuse_next && m.tensors[q.dst].h == (m.tensors[c.dst].h - 1) / 2 + 1 &&
            m.tensors[q.dst].w == (m.tensors[c.dst].w - 1) / 2 + 1) {
            m.ops[stem_op].fuse_pool = true;
            m.tensors[q.dst].def = std::min(m.tensors[q.dst].def, stem_op);
        }
    }
    if (stem_op >= 0) {                                          // tensor 0 as the staging kernel writes it
        m.stem_s2d = true;
        TensorInfo& t0 = m.tensors[0];
        t0.h = (t0.h + 1) / 2; t0.w = (t0.w + 1) / 2; t0.c = 12; t0.cs = 16;
    }
    m.tensors[spec.out_tensor].external = true;
    bw.reserve(0);
    m.host_params.resize(align_up(m.host_params.size()), 0);
    *out = std::move(m);
    return ENS_OK;
}

// Lowest-offset placement of every tensor among the tensors alive at the same time.
ArenaLayout plan_arena(const Member& m, int batch, bool keep_all) {
    ArenaLayout L;
    const int NT = (int)m.tensors.size();
    L.offset.assign(NT, 0);
    std::vector<int> order;
    for (int t = 0; t < NT; t++)
        if (!m.tensors[t].external && m.tensors[t].def != INT32_MAX) order.push_back(t);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return m.tensors[a].def < m.tensors[b].def; });
    std::vector<int> placed;
    for (int t : order) {
        const TensorInfo& ti = m.tensors[t];
        const size_t need = align_up(ti.bytes(batch));
        const int last = std::max(ti.last, ti.def);
        std::vector<std::pair<size_t, size_t>> busy;
        for (int u : placed) {
            const TensorInfo& tu = m.tensors[u];
            const int ulast = std::max(tu.last, tu.def);
            if (keep_all || (tu.def <= last && ti.def <= ulast)) busy.push_back({L.offset[u], L.offset[u] + align_up(tu.bytes(batch))});
        }
        std::sort(busy.begin(), busy.end());
        size_t off = 0;
        for (const auto& iv : busy) {
            if (off + need <= iv.first) break;
            off = std::max(off, iv.second);
        }
        L.offset[t] = off;
        L.bytes = std::max(L.bytes, off + need);
        placed.push_back(t);
    }
    if (m.bf16) {                      // split-K workspace and tickets of the convolution kernel
        L.scratch_offset = align_up(L.bytes);
        L.bytes = L.scratch_offset + align_up(SPLIT_WS_FLOATS * sizeof(float));
    }
    return L;
}

}  // namespace ens
