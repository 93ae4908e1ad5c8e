/*
 * CPU oracle of an ensemble member's forward pass.  TEST INFRASTRUCTURE ONLY:
 * a plain, slow, direct implementation used to check the GPU library; nothing
 * on the product path may call it, and it shares no code with that path.
 *
 * The paper delegates the member forward pass ("predictor", section "The worker
 * pool") to an inference framework; what a member computes is fixed by its
 * operation list (convolution, depthwise convolution, pooling, squeeze-excite,
 * fully connected), each written here from its textbook definition as nested
 * loops over one image at a time, with no blocking, fusion or reordering.
 *
 * Arithmetic type REAL is float (the reference precision of the workloads) or
 * double (compile with -DREAL=double) for cross-checks of rounding error.
 * Batch-norm is applied unfolded: gamma * (x - mean) / sqrt(var + eps) + beta.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL float
#endif

#define BN_EPS 1e-5

enum { OP_CONV = 1, OP_DWCONV = 2, OP_MAXPOOL = 3, OP_AVGPOOL = 4, OP_GAP = 5, OP_FC = 6, OP_SE = 7 };
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_SILU = 2 };

typedef struct {
    int32_t kind, src, src_c0, cin, dst, dst_c0, cout;
    int32_t kh, kw, sh, sw, pt, pl, act, res, res_c0, pre, r;
    int64_t off_w, off_b, off_bn, off_pre, off_w2, off_b2;
} orc_op;

typedef struct { int32_t h, w, c; } orc_tensor;

static REAL act_fn(REAL x, int act) {
    if (act == ACT_RELU) return x > 0 ? x : 0;
    if (act == ACT_SILU) return x / (1 + (REAL)exp(-(double)x));
    return x;
}

/* round to nearest-even bf16, returned widened (diagnostic storage mode) */
static REAL round_bf16(REAL v) {
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return (REAL)f;
}

static REAL bn_apply(REAL x, const float* bn, int c, int C) {
    /* bn = [gamma(C), beta(C), mean(C), var(C)] */
    REAL g = bn[c], b = bn[C + c], m = bn[2 * C + c], v = bn[3 * C + c];
    return g * (x - m) / (REAL)sqrt((double)v + BN_EPS) + b;
}

static void conv_op(const orc_op* o, const orc_tensor* T, REAL** buf, const float* blob) {
    const orc_tensor ti = T[o->src], to = T[o->dst];
    const REAL* in = buf[o->src];
    REAL* out = buf[o->dst];
    const float* w = blob + o->off_w;
    REAL* acc = (REAL*)malloc(sizeof(REAL) * o->cout);
    const int groups = o->r > 1 ? o->r : 1;          /* CONV: r = number of groups (0 or 1: ordinary) */
    const int ig = o->cin / groups, og = o->cout / groups;
    for (int ho = 0; ho < to.h; ho++)
        for (int wo = 0; wo < to.w; wo++) {
            for (int co = 0; co < o->cout; co++) acc[co] = 0;
            for (int kh = 0; kh < o->kh; kh++) {
                int hi = ho * o->sh - o->pt + kh;
                if (hi < 0 || hi >= ti.h) continue;
                for (int kw = 0; kw < o->kw; kw++) {
                    int wi = wo * o->sw - o->pl + kw;
                    if (wi < 0 || wi >= ti.w) continue;
                    const REAL* px = in + ((size_t)hi * ti.w + wi) * ti.c + o->src_c0;
                    /* groups: output channel co belongs to group co / og and sees only that group's
                       ig input channels; the weights are [kh][kw][ig][cout] */
                    const float* wk = w + (size_t)(kh * o->kw + kw) * ig * o->cout;
                    for (int ci = 0; ci < o->cin; ci++) {
                        REAL x = px[ci];
                        if (o->pre) {
                            x = bn_apply(x, blob + o->off_pre, ci, o->cin);
                            x = x > 0 ? x : 0;
                        }
                        const int g = ci / ig;
                        const float* wr = wk + (size_t)(ci - g * ig) * o->cout;
                        for (int co = g * og; co < (g + 1) * og; co++) acc[co] += x * (REAL)wr[co];
                    }
                }
            }
            REAL* po = out + ((size_t)ho * to.w + wo) * to.c + o->dst_c0;
            for (int co = 0; co < o->cout; co++) {
                REAL y = acc[co];
                if (o->off_b >= 0) y += (REAL)blob[o->off_b + co];
                if (o->off_bn >= 0) y = bn_apply(y, blob + o->off_bn, co, o->cout);
                if (o->res >= 0)
                    y += buf[o->res][((size_t)ho * to.w + wo) * T[o->res].c + o->res_c0 + co];
                po[co] = act_fn(y, o->act);
            }
        }
    free(acc);
}

static void dwconv_op(const orc_op* o, const orc_tensor* T, REAL** buf, const float* blob) {
    const orc_tensor ti = T[o->src], to = T[o->dst];
    const REAL* in = buf[o->src];
    REAL* out = buf[o->dst];
    const float* w = blob + o->off_w; /* [kh][kw][c] */
    for (int ho = 0; ho < to.h; ho++)
        for (int wo = 0; wo < to.w; wo++)
            for (int c = 0; c < o->cin; c++) {
                REAL acc = 0;
                for (int kh = 0; kh < o->kh; kh++) {
                    int hi = ho * o->sh - o->pt + kh;
                    if (hi < 0 || hi >= ti.h) continue;
                    for (int kw = 0; kw < o->kw; kw++) {
                        int wi = wo * o->sw - o->pl + kw;
                        if (wi < 0 || wi >= ti.w) continue;
                        acc += in[((size_t)hi * ti.w + wi) * ti.c + o->src_c0 + c] *
                               (REAL)w[(size_t)(kh * o->kw + kw) * o->cin + c];
                    }
                }
                if (o->off_b >= 0) acc += (REAL)blob[o->off_b + c];
                if (o->off_bn >= 0) acc = bn_apply(acc, blob + o->off_bn, c, o->cin);
                out[((size_t)ho * to.w + wo) * to.c + o->dst_c0 + c] = act_fn(acc, o->act);
            }
}

static void pool_op(const orc_op* o, const orc_tensor* T, REAL** buf) {
    const orc_tensor ti = T[o->src], to = T[o->dst];
    const REAL* in = buf[o->src];
    REAL* out = buf[o->dst];
    for (int ho = 0; ho < to.h; ho++)
        for (int wo = 0; wo < to.w; wo++)
            for (int c = 0; c < o->cin; c++) {
                REAL m = 0, s = 0;
                int cnt = 0;
                for (int kh = 0; kh < o->kh; kh++) {
                    int hi = ho * o->sh - o->pt + kh;
                    if (hi < 0 || hi >= ti.h) continue;
                    for (int kw = 0; kw < o->kw; kw++) {
                        int wi = wo * o->sw - o->pl + kw;
                        if (wi < 0 || wi >= ti.w) continue;
                        REAL x = in[((size_t)hi * ti.w + wi) * ti.c + o->src_c0 + c];
                        if (cnt == 0 || x > m) m = x;
                        s += x;
                        cnt++;
                    }
                }
                out[((size_t)ho * to.w + wo) * to.c + o->dst_c0 + c] =
                    o->kind == OP_MAXPOOL ? m : (cnt ? s / (REAL)cnt : 0);
            }
}

static void gap_op(const orc_op* o, const orc_tensor* T, REAL** buf, const float* blob) {
    const orc_tensor ti = T[o->src];
    const REAL* in = buf[o->src];
    REAL* out = buf[o->dst];
    for (int c = 0; c < o->cin; c++) {
        REAL s = 0;
        for (int p = 0; p < ti.h * ti.w; p++) {
            REAL x = in[(size_t)p * ti.c + o->src_c0 + c];
            if (o->pre) {
                x = bn_apply(x, blob + o->off_pre, c, o->cin);
                x = x > 0 ? x : 0;
            }
            s += x;
        }
        out[o->dst_c0 + c] = s / (REAL)(ti.h * ti.w);
    }
}

static void fc_op(const orc_op* o, REAL** buf, const float* blob) {
    const REAL* in = buf[o->src] + o->src_c0;
    REAL* out = buf[o->dst] + o->dst_c0;
    const float* w = blob + o->off_w; /* [cin][cout] */
    for (int co = 0; co < o->cout; co++) {
        REAL s = 0;
        for (int ci = 0; ci < o->cin; ci++) s += in[ci] * (REAL)w[(size_t)ci * o->cout + co];
        out[co] = s + (REAL)blob[o->off_b + co];
    }
}

static void se_op(const orc_op* o, const orc_tensor* T, REAL** buf, const float* blob) {
    const orc_tensor ti = T[o->src];
    const REAL* in = buf[o->src];
    REAL* out = buf[o->dst];
    int C = o->cin, R = o->r, P = ti.h * ti.w;
    REAL* s = (REAL*)malloc(sizeof(REAL) * (C + R + C));
    REAL* z = s + C;
    REAL* g = z + R;
    for (int c = 0; c < C; c++) {
        REAL a = 0;
        for (int p = 0; p < P; p++) a += in[(size_t)p * ti.c + o->src_c0 + c];
        s[c] = a / (REAL)P;
    }
    for (int r = 0; r < R; r++) {
        REAL a = 0;
        for (int c = 0; c < C; c++) a += s[c] * (REAL)blob[o->off_w + (size_t)c * R + r];
        z[r] = act_fn(a + (REAL)blob[o->off_b + r], ACT_SILU);
    }
    for (int c = 0; c < C; c++) {
        REAL a = 0;
        for (int r = 0; r < R; r++) a += z[r] * (REAL)blob[o->off_w2 + (size_t)r * C + c];
        a += (REAL)blob[o->off_b2 + c];
        g[c] = 1 / (1 + (REAL)exp(-(double)a));
    }
    for (int p = 0; p < P; p++)
        for (int c = 0; c < C; c++)
            out[(size_t)p * T[o->dst].c + o->dst_c0 + c] = in[(size_t)p * ti.c + o->src_c0 + c] * g[c];
    free(s);
}

/*
 * Forward pass of one member over n images.
 *   images : n x H x W x C fp32 (tensor 0 of the description)
 *   out    : n x size(out_tensor) doubles (the logits)
 *   store_bf16 != 0 : diagnostic mode, every image-shaped operation output is
 *                     rounded to bf16 where a bf16 pipeline would store it
 *   dump_tensor >= 0: additionally copy that tensor of image 0 into dump (doubles)
 * Returns 0, or -1 on a malformed description.
 */
int orc_forward(const orc_tensor* T, int n_tensors, const orc_op* ops, int n_ops, const float* blob,
                const float* images, int n, int out_tensor, double* out, int store_bf16,
                int dump_tensor, double* dump) {
    if (out_tensor < 0 || out_tensor >= n_tensors) return -1;
    for (int i = 0; i < n_ops; i++) {
        const orc_op* o = &ops[i];
        if (o->src < 0 || o->src >= n_tensors || o->dst < 0 || o->dst >= n_tensors) return -1;
        if (o->src_c0 + o->cin > T[o->src].c || o->dst_c0 + o->cout > T[o->dst].c) return -1;
        if (o->res >= n_tensors) return -1;
    }
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int img = 0; img < n; img++) {
        REAL** buf = (REAL**)calloc(n_tensors, sizeof(REAL*));
        for (int t = 0; t < n_tensors; t++) {
            size_t sz = (size_t)T[t].h * T[t].w * T[t].c;
            buf[t] = (REAL*)calloc(sz, sizeof(REAL));
            if (!buf[t]) failed = 1;
        }
        if (!failed) {
            size_t isz = (size_t)T[0].h * T[0].w * T[0].c;
            for (size_t e = 0; e < isz; e++) buf[0][e] = (REAL)images[(size_t)img * isz + e];
            for (int i = 0; i < n_ops; i++) {
                const orc_op* o = &ops[i];
                switch (o->kind) {
                    case OP_CONV: conv_op(o, T, buf, blob); break;
                    case OP_DWCONV: dwconv_op(o, T, buf, blob); break;
                    case OP_MAXPOOL:
                    case OP_AVGPOOL: pool_op(o, T, buf); break;
                    case OP_GAP: gap_op(o, T, buf, blob); break;
                    case OP_FC: fc_op(o, buf, blob); break;
                    case OP_SE: se_op(o, T, buf, blob); break;
                    default: failed = 1;
                }
                if (store_bf16 && o->kind != OP_GAP && o->kind != OP_FC) {
                    const orc_tensor to = T[o->dst];
                    for (size_t p = 0; p < (size_t)to.h * to.w; p++)
                        for (int c = 0; c < o->cout; c++) {
                            REAL* q = &buf[o->dst][p * to.c + o->dst_c0 + c];
                            *q = round_bf16(*q);
                        }
                }
            }
            size_t osz = (size_t)T[out_tensor].h * T[out_tensor].w * T[out_tensor].c;
            for (size_t e = 0; e < osz; e++) out[(size_t)img * osz + e] = (double)buf[out_tensor][e];
            if (img == 0 && dump_tensor >= 0 && dump_tensor < n_tensors) {
                size_t dsz = (size_t)T[dump_tensor].h * T[dump_tensor].w * T[dump_tensor].c;
                for (size_t e = 0; e < dsz; e++) dump[e] = (double)buf[dump_tensor][e];
            }
        }
        for (int t = 0; t < n_tensors; t++) free(buf[t]);
        free(buf);
    }
    return failed ? -1 : 0;
}

int orc_real_bytes(void) { return (int)sizeof(REAL); }
