"""An interpreter of the member operation lists on top of PyTorch's CPU library
routines in fp64.  Used only to pin the C oracle: conv2d / pooling / matmul here
are library code that shares nothing with the oracle's nested loops."""
import numpy as np
import torch
import torch.nn.functional as F
from synth import nets as N


def _bn(x, p, C):
    g, b, m, v = p[:C], p[C:2 * C], p[2 * C:3 * C], p[3 * C:4 * C]
    sh = (1, C, 1, 1)
    return g.view(sh) * (x - m.view(sh)) / torch.sqrt(v.view(sh) + N.BN_EPS) + b.view(sh)


def _act(x, a):
    if a == N.ACT_RELU:
        return torch.relu(x)
    if a == N.ACT_SILU:
        return x * torch.sigmoid(x)
    return x


def run(net, blob, images, want=None):
    """Returns logits (n x classes); with `want` a tensor id returns that tensor (NHWC)."""
    blob = torch.from_numpy(np.asarray(blob, dtype=np.float64))
    x0 = torch.from_numpy(np.asarray(images, dtype=np.float64)).permute(0, 3, 1, 2)
    n = x0.shape[0]
    T = [None] * len(net.tensors)
    T[0] = x0

    def ensure(t):
        if T[t] is None:
            h, w, c = net.tensors[t]
            T[t] = torch.zeros(n, c, h, w, dtype=torch.float64)
        return T[t]

    for o in net.ops:
        k = o["kind"]
        src = T[o["src"]][:, o["src_c0"]:o["src_c0"] + o["cin"]]
        ho, wo, _ = net.tensors[o["dst"]]
        dst = ensure(o["dst"])
        sl = slice(o["dst_c0"], o["dst_c0"] + o["cout"])
        if k in (N.CONV, N.DWCONV):
            if o["pre"]:
                src = torch.relu(_bn(src, blob[o["off_pre"]:o["off_pre"] + 4 * o["cin"]], o["cin"]))
            kh, kw, cin, cout = o["kh"], o["kw"], o["cin"], o["cout"]
            if k == N.CONV:
                groups = max(1, o["r"])                          # CONV: r = number of groups
                ig = cin // groups
                w = blob[o["off_w"]:o["off_w"] + kh * kw * ig * cout].view(kh, kw, ig, cout).permute(3, 2, 0, 1)
            else:
                w = blob[o["off_w"]:o["off_w"] + kh * kw * cin].view(kh, kw, 1, cin).permute(3, 2, 0, 1)
                groups = cin
            h, wd = src.shape[2], src.shape[3]
            pb = max(0, (ho - 1) * o["sh"] + kh - o["pt"] - h)
            pr = max(0, (wo - 1) * o["sw"] + kw - o["pl"] - wd)
            xp = F.pad(src, (o["pl"], pr, o["pt"], pb))
            y = F.conv2d(xp, w.contiguous(), stride=(o["sh"], o["sw"]), groups=groups)[:, :, :ho, :wo]
            if o["off_b"] >= 0:
                y = y + blob[o["off_b"]:o["off_b"] + cout].view(1, cout, 1, 1)
            if o["off_bn"] >= 0:
                y = _bn(y, blob[o["off_bn"]:o["off_bn"] + 4 * cout], cout)
            if o["res"] >= 0:
                y = y + T[o["res"]][:, o["res_c0"]:o["res_c0"] + cout]
            dst[:, sl] = _act(y, o["act"])
        elif k in (N.MAXPOOL, N.AVGPOOL):
            kk, s, p = o["kh"], o["sh"], o["pt"]
            if k == N.MAXPOOL:
                y = F.max_pool2d(src, kk, s, p)
            else:
                y = F.avg_pool2d(src, kk, s, p, count_include_pad=False)
            dst[:, sl] = y[:, :, :ho, :wo]
        elif k == N.GAP:
            if o["pre"]:
                src = torch.relu(_bn(src, blob[o["off_pre"]:o["off_pre"] + 4 * o["cin"]], o["cin"]))
            dst[:, sl] = src.mean(dim=(2, 3), keepdim=True)
        elif k == N.FC:
            w = blob[o["off_w"]:o["off_w"] + o["cin"] * o["cout"]].view(o["cin"], o["cout"])
            y = src.reshape(n, o["cin"]) @ w + blob[o["off_b"]:o["off_b"] + o["cout"]]
            dst[:, sl] = y.view(n, o["cout"], 1, 1)
        elif k == N.SE:
            C, R = o["cin"], o["r"]
            s = src.mean(dim=(2, 3))
            w1 = blob[o["off_w"]:o["off_w"] + C * R].view(C, R)
            z = s @ w1 + blob[o["off_b"]:o["off_b"] + R]
            z = z * torch.sigmoid(z)
            w2 = blob[o["off_w2"]:o["off_w2"] + R * C].view(R, C)
            g = torch.sigmoid(z @ w2 + blob[o["off_b2"]:o["off_b2"] + C])
            dst[:, sl] = src * g.view(n, C, 1, 1)
        else:
            raise ValueError(k)
    t = net.out_tensor if want is None else want
    out = T[t].permute(0, 2, 3, 1).contiguous().numpy()
    return out.reshape(n, -1) if want is None else out
