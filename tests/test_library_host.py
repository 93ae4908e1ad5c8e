"""Host-side checks of the GPU library that need no GPU: the C interface loads and exports
what include/ens.h declares, and the C++ planner / partition / memory model agree with the
oracle's literal Algorithms 1 and 2 on the same inputs."""
import ctypes
import os
import random
import re

import pytest

import oracle
from oracle import planner as P
import paper_2208_14049_amd as ens
from synth import nets as N

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ens.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ens_[a-z_0-9]+)\s*\(", header))
    declared -= {"ens_bench_fn", "ens_bench_single_fn"}
    assert len(declared) >= 20
    L = ens.lib()
    for name in sorted(declared):
        assert hasattr(L, name), name
    assert set(ens.EXPORTS) == declared
    assert b"gfx950" in L.ens_version()
    assert L.ens_strerror(ens.ENS_E_NOFIT) != L.ens_strerror(ens.ENS_E_NOMEM)


def random_problem(rnd, pooled=False):
    M = rnd.randint(1, 4)
    R = rnd.randint(1, 4)
    domain = [8, 16, 32]
    weights = [rnd.randint(1, 40) for _ in range(M)]
    arena = [[rnd.randint(1, 10) * b // 8 for b in domain] for _ in range(M)]
    if pooled:
        row_pool, caps = [0] * R, [rnd.randint(30, 200)]
    else:
        row_pool, caps = list(range(R)), [rnd.randint(10, 90) for _ in range(R)]
    kinds = [rnd.random() < 0.7 for _ in range(R)]
    return M, R, domain, weights, arena, row_pool, kinds, caps


def both(M, R, domain, weights, arena, row_pool, kinds, caps, **kw):
    prob = ens.PlanProblem(weights, arena, domain, 8, row_pool, kinds, caps, **kw)
    mem = P.Memory(weights, lambda m, b: arena[m][domain.index(b)], row_pool,
                   ["GPU" if k else "CPU" for k in kinds], caps)
    return prob, mem


def test_wfd_matches_oracle_on_random_instances():
    rnd = random.Random(1)
    n_fail = n_ok = 0
    for it in range(300):
        args = random_problem(rnd, pooled=(it % 3 == 0))
        prob, mem = both(*args)
        try:
            exp = P.worst_fit_decreasing(args[0], mem, 8)
        except MemoryError:
            exp = None
        if exp is None:
            with pytest.raises(ens.EnsError) as e:
                prob.wfd()
            assert e.value.status == ens.ENS_E_NOFIT
            n_fail += 1
        else:
            got = prob.wfd()
            assert got == exp
            assert prob.fit_mem(got) and P.fit_mem(exp, mem)
            n_ok += 1
    assert n_fail > 10 and n_ok > 50


def test_fit_mem_and_neighbors_match_oracle():
    rnd = random.Random(2)
    for it in range(100):
        M, R, domain, weights, arena, row_pool, kinds, caps = random_problem(rnd, pooled=(it % 2 == 0))
        prob, mem = both(M, R, domain, weights, arena, row_pool, kinds, caps)
        A = [[rnd.choice([0] + domain) for _ in range(M)] for _ in range(R)]
        assert prob.fit_mem(A) == P.fit_mem(A, mem)
        if P.is_valid(A):
            assert prob.neighbors(A) == P.neighborhood(A, domain)
        else:
            with pytest.raises(ens.EnsError):
                prob.neighbors(A)


def test_greedy_matches_oracle_with_injected_cost_model():
    rnd = random.Random(3)
    for it in range(40):
        M, R, domain, weights, arena, row_pool, kinds, caps = random_problem(rnd, pooled=True)
        caps = [10 ** 6]
        table = {}
        seed_cost = rnd.randint(0, 10 ** 6)

        def bench(A):
            key = tuple(map(tuple, A))
            if key not in table:
                table[key] = random.Random(hash(key) ^ seed_cost).random()
            return table[key]

        max_iter, max_neighs, seed = rnd.randint(1, 6), rnd.choice([3, 10, 1000]), rnd.randint(0, 2 ** 40)
        prob, mem = both(M, R, domain, weights, arena, row_pool, kinds, caps,
                         max_iter=max_iter, max_neighs=max_neighs, seed=seed)
        start = P.worst_fit_decreasing(M, mem, 8)
        exp_a, exp_s, exp_n = P.bounded_greedy(start, bench, domain, max_iter, max_neighs, seed)
        got_a, got_s, got_n = prob.greedy(start, bench)
        assert (got_a, got_n) == (exp_a, exp_n)
        assert got_s == exp_s >= bench(start)


def test_bbs_matches_oracle():
    domain = [8, 16, 32, 64, 128]
    prob = ens.PlanProblem([1] * 4, [[1] * 5] * 4, domain, 8, [0], [1], [10 ** 9])
    speed = lambda m, b: -abs(b - [8, 32, 128, 64][m])
    got, n = prob.bbs(speed)
    exp, n2 = P.best_batch_size(4, speed, domain)
    assert got == exp == [8, 32, 128, 64] and n == n2 == 20


@pytest.mark.parametrize("n,seg,b", [(300, 128, 8), (300, 128, 128), (1024, 128, 32), (1, 128, 8), (0, 128, 8),
                                      (129, 128, 64), (2048, 256, 256), (77, 16, 5)])
def test_partition_matches_oracle(n, seg, b):
    exp = [bt for (a, e) in oracle.segments(n, seg) for bt in oracle.batches(a, e, b)]
    assert ens.ens_partition(n, seg, b) == exp


def test_hand_out_matches_oracle_queue_simulation():
    """The library decides on the host which worker of a member takes which segment; the oracle runs the
    shared FIFO queue of section "Data-parallelism" as an event simulation in the same model of time."""
    rnd = random.Random(11)
    for _ in range(200):
        k = rnd.randint(1, 6)
        b = [rnd.choice([1, 4, 8, 16, 32, 64, 128, 256]) for _ in range(k)]
        n, seg = rnd.randint(0, 5000), rnd.choice([16, 64, 128, 256])
        lc, ic = rnd.choice([0.0, 1e-4, 4e-4]), rnd.choice([0.0, 1e-5, 5e-5])
        assert ens.ens_hand_out(n, seg, b, lc, ic) == oracle.fifo_hand_out(n, seg, b, lc, ic), (n, seg, b, lc, ic)
    assert ens.ens_hand_out(128 * 5, 128, [32, 32], 3e-4, 2e-5) == [0, 1, 0, 1, 0]


def test_memory_model_from_description():
    net = N.resnet18()
    w, a8 = ens.ens_spec_bytes(net, 8)
    _, a32 = ens.ens_spec_bytes(net, 32)
    n_w = sum(p["size"] for p in net.params if p["role"] == "conv_w")
    # bf16 weights; the FC head once more, transposed, in matrix-core operand order (1000 rows padded to 1024);
    # fp32 bias and scale per output channel; alignment; the stem's filter padded to 16 channels per tap
    fc_copy = 2 * 1024 * 512
    # and the three strided 1x1 shortcuts once more in operand order (rows in 32s, input channels in 64s)
    fc_copy += 2 * (128 * 64 + 256 * 128 + 512 * 256)
    assert 2 * n_w + fc_copy <= w <= 2 * n_w + fc_copy + 2 * 4 * 20000 + 256 * 4 * len(net.ops) + 2 * 8 * 64 * 49
    # the arena is at least the two largest tensors alive together (stem output and its input, which
    # a bf16 member stores space-to-depth: 112 x 112 pixels of 16 channels)
    stem_in, stem_out = 112 * 112 * 16 * 2, 112 * 112 * 64 * 2
    scratch = (4 << 20) * 4                      # split-K workspace of a bf16 worker
    assert a8 - scratch >= 8 * (stem_in + stem_out)
    assert a8 - scratch <= 8 * (stem_in + 3 * stem_out)
    assert abs((a32 - scratch) / (a8 - scratch) - 4.0) < 0.05
    tiny = N.tiny_a()
    w, a = ens.ens_spec_bytes(tiny, 8)
    assert w >= 4 * (432 + 16 + 4608 + 32 + 320 + 10)
    assert a >= 8 * 4 * (32 * 32 * 3 + 32 * 32 * 16)


def test_load_reports_missing_gpu_or_succeeds():
    import torch
    nets = N.config_members(1)
    if torch.cuda.is_available():
        pytest.skip("a GPU is present; covered by the gpu tests")
    with pytest.raises(ens.EnsError) as e:
        ens.Ensemble(nets, seed=1)
    assert e.value.status == ens.ENS_E_NODEVICE


def test_invalid_descriptions_are_rejected():
    net = N.tiny_a()
    net.ops[0]["off_w"] = net.blob_size        # weights beyond the blob
    with pytest.raises(ens.EnsError) as e:
        ens.ens_spec_bytes(net, 8)
    assert e.value.status == ens.ENS_E_INVALID
    net = N.Net("odd", 16, 16, 10, dtype="bf16")
    t = net.conv(0, 12, 3)                       # 12 output channels: not a multiple of 8
    net.fc(net.gap(t), 10)
    with pytest.raises(ens.EnsError) as e:
        ens.ens_spec_bytes(net, 8)
    assert e.value.status == ens.ENS_E_UNSUPPORTED


def test_grouped_convolutions_in_descriptions():
    """The plan accepts the grouped layers of the ResNeXt shape (its weights are the dense 32-channel
    blocks, so the parameter block grows with the zeros between groups) and rejects group counts that
    do not divide the channels, groups that do not tile a 32-channel block, and fp32 members."""
    net = N.resnext50()
    w, _ = ens.ens_spec_bytes(net, 8)
    n_w = sum(p["size"] for p in net.params if p["role"] == "conv_w")
    dense_blocks = sum(9 * op["cout"] * 32 for op in net.ops if op["kind"] == N.CONV and op["r"] > 1)
    grouped = sum(9 * op["cout"] * op["cin"] // op["r"] for op in net.ops if op["kind"] == N.CONV and op["r"] > 1)
    # plus the second, operand-ordered copy of the 1x1 layers (padding 0) that a kernel fetches straight from memory
    copies = sum(-(-op["cin"] // 64) * 64 * -(-op["cout"] // 32) * 32 for op in net.ops
                 if op["kind"] == N.CONV and op["kh"] == 1 and op["kw"] == 1 and op["r"] <= 1)
    assert copies > 0
    copies += 1024 * 2048                                        # the FC head once more, transposed, 1000 rows padded to 1024
    expected = 2 * (n_w - grouped + dense_blocks + copies)
    assert expected <= w <= expected + 2 * 4 * 40000 + 1024 * len(net.ops)    # + fp32 bias and scale per output channel, alignment

    def one(cin, cout, groups, dtype="bf16"):
        n = N.Net("g", 16, 16, 10, dtype=dtype)
        t = n.conv(0, cin, 1)
        t = n.conv(t, cout, 3, groups=groups)
        n.fc(n.gap(t), 10)
        return n

    ens.ens_spec_bytes(one(64, 64, 4), 8)                       # 16 per group: two groups per block
    ens.ens_spec_bytes(one(128, 256, 2), 8)                     # groups wider than a block
    for bad, status in ((one(96, 96, 8), ens.ENS_E_UNSUPPORTED),          # 12 per group does not divide 32
                        (one(64, 64, 4, dtype="fp32"), ens.ENS_E_UNSUPPORTED)):
        with pytest.raises(ens.EnsError) as e:
            ens.ens_spec_bytes(bad, 8)
        assert e.value.status == status
    bad = one(64, 64, 4)
    bad.ops[1]["r"] = 5                                          # 5 groups do not divide 64 channels
    with pytest.raises(ens.EnsError) as e:
        ens.ens_spec_bytes(bad, 8)
    assert e.value.status == ens.ENS_E_INVALID


def test_dense_block_layers_in_descriptions():
    """A layer of a dense block that one kernel can run (pre-activated 1x1 to 128 channels, 3x3 to 32
    channels appended to the block's tensor, nobody else reading the tensor in between) gets operand-
    ordered copies of both filters; with a second reader of the middle tensor it gets none.  The two
    networks below hold the same layers with the same parameter sizes and differ only in what the
    extra 1x1 layer reads."""
    def net(tap_middle):
        n = N.Net("d", 12, 12, 8, dtype="bf16")
        blk = n.tensor(12, 12, 128 + 32)
        n.conv(0, 128, 3, dst=(blk, 0))
        u = n.conv(blk, 128, 1, pre=True, src_slice=(0, 128))
        n.conv(u, 32, 3, bn=False, act=None, bias=False, dst=(blk, 128))
        if tap_middle:
            t = n.conv(u, 8, 1)
        else:
            t = n.conv(blk, 8, 1, src_slice=(0, 128))
        n.fc(n.gap(t), 8)
        return n

    up = lambda b: (b + 255) // 256 * 256
    fused, _ = ens.ens_spec_bytes(net(False), 8)
    plain, _ = ens.ens_spec_bytes(net(True), 8)
    assert fused - plain == up(2 * 128 * 128) + up(2 * 9 * 128 * 32), fused - plain


def test_transition_convolution_gets_an_operand_ordered_copy():
    """The pre-activated 1x1 convolution of a transition (no activation, its output read by a 2x2 / stride-2 average
    pool alone) can run behind that pool as a plain 1x1 layer: the plan gives it the second, operand-ordered copy of
    its weights that the weights-from-memory kernel reads (input channels padded to 64, output channels to 32).
    With a max-pool behind it, an activation of its own, or a second reader of its output it gets none."""
    def net(pool, act=None, tap=False):
        n = N.Net("tr", 16, 16, 8, dtype="bf16")
        x = n.conv(0, 96, 3)
        u = n.conv(x, 40, 1, pre=True, bn=False, act=act, bias=False)
        t = n.avgpool(u, 2, 2) if pool == "avg" else n.maxpool(u, 2, 2)
        t2 = n.conv(u, 8, 3, stride=2) if tap else None            # a second reader of the convolution's output
        v = n.conv(t, 8, 3, res=t2)
        n.fc(n.gap(v), 8)
        return n

    up = lambda b: (b + 255) // 256 * 256
    swapped, _ = ens.ens_spec_bytes(net("avg"), 8)
    plain, _ = ens.ens_spec_bytes(net("max"), 8)
    assert swapped - plain == up(2 * 128 * 64), swapped - plain     # 96 -> 128 input channels, 40 -> 64 output channels
    with_act, _ = ens.ens_spec_bytes(net("avg", act="relu"), 8)
    assert with_act == plain
    a, _ = ens.ens_spec_bytes(net("avg", tap=True), 8)
    b, _ = ens.ens_spec_bytes(net("max", tap=True), 8)
    assert a == b


def test_squeeze_excite_scratch_behind_a_depthwise_layer():
    """A squeeze-excite block behind a 3x3 or 5x5 depthwise layer (bf16) gets the channel sums from that layer's
    kernel, one row per workgroup of an image: its scratch holds as many rows as that kernel has workgroups per
    image (never fewer than the block's own kernel writes) and is live from the depthwise layer on.  A 7x7
    depthwise layer, which that kernel does not run, leaves the block's scratch as it is.  (That the rows are
    enough is checked where the kernel runs: the engine takes the summing kernel only when they are.)"""
    def net(h, c, k):
        n = N.Net("dwse", h, h, 8, dtype="bf16")
        t = n.conv(0, c, 1, act="silu")
        u = n.se(n.dwconv(t, k, 1), 4)
        n.fc(n.gap(u), 8)
        return n

    batch = 8
    for h, c in ((112, 32), (56, 144), (14, 480)):
        rows = max(16, -(-(h * -(-h // 4) * (c // 8)) // 256))   # 256 lanes of 4 columns x 8 channels
        for k in (3, 5):
            _, fused = ens.ens_spec_bytes(net(h, c, k), batch)
            _, plain = ens.ens_spec_bytes(net(h, c, 7), batch)
            # the arena grows by the extra rows at most (by less where the scratch fits a gap that the packing leaves)
            assert 0 <= fused - plain <= batch * (rows - 16) * c * 4 + 256, (h, c, k, fused - plain, rows)
    assert rows == 16 and fused == plain                         # 14x14x480: 14 workgroups, the scratch stays at 16 rows


def test_dense_layer_output_does_not_share_memory_with_its_input():
    """A pre-activated 1x1 (to 128 channels) followed by a 3x3 (to 32) may run as one kernel that writes the
    3x3's output while other workgroups still read the 1x1's input: when the output is a tensor of its own it
    must not be placed over that input, although the input's last reader is the first of the two operations."""
    n = N.Net("dl", 16, 16, 8, dtype="bf16")
    a = n.conv(0, 64, 3)
    u = n.conv(a, 128, 1, pre=True)
    c = n.conv(u, 32, 3, bn=False, act=None, bias=False)
    n.fc(n.gap(c), 8)
    batch = 4
    _, arena = ens.ens_spec_bytes(n, batch)
    px = batch * 16 * 16 * 2
    workspace = 16 << 20                                         # split-K workspace appended to a bf16 worker's arena
    assert arena - workspace >= px * (64 + 128 + 32)             # input, middle and output alive together


def test_bottleneck_chains_in_descriptions():
    """The plan keeps a second copy, in matrix-core operand order (rows padded to 32, columns to 64), of
    the weights of layers that kernels fetch straight from memory: every 1x1 convolution without padding
    or pre-activation, and the 3x3 layer of a residual bottleneck that one kernel can run (1x1, 3x3
    stride 1, 1x1, with 64 or 128 channels in between and nobody else touching the two middle
    tensors).  The parameter block grows by exactly those copies: the same layers with a stride on the
    3x3, another width in the middle, a second reader of a middle tensor or fp32 parameters get no
    copy of the 3x3 filter."""
    def block(c, cin, cout, stride=1, tap_t1=False, dtype="bf16"):
        n = N.Net("b", 16, 16, 10, dtype=dtype)
        x = n.conv(0, cin, 3)
        t1 = n.conv(x, c, 1)
        t2 = n.conv(t1, c, 3, stride=stride)
        y = n.conv(t2, cout, 1)
        g = n.gap(y)
        if tap_t1:
            n.conv(t1, 8, 1)                                     # someone else reads the first middle tensor
        n.fc(g, 10)
        return n

    up = lambda b: (b + 255) // 256 * 256
    pointwise = lambda cin, cout: up(2 * (-(-cin // 64) * 64) * (-(-cout // 32) * 32))

    for c, cin, cout in ((64, 256, 256), (128, 64, 512), (64, 32, 128)):
        fused, _ = ens.ens_spec_bytes(block(c, cin, cout), 8)
        plain, _ = ens.ens_spec_bytes(block(c, cin, cout, stride=2), 8)
        assert fused - plain == up(2 * 9 * c * c), (c, cin, cout, fused - plain)
    # the 1x1 layers alone: a layer without padding gets the padded copy (256 -> 64 as it is; 40 -> 24 as 64 -> 32) at
    # stride 1 and at stride 2 (the shortcuts of residual stages), a pre-activated one none
    for cin, cout in ((256, 64), (40, 24)):
        n1 = N.Net("p", 16, 16, 10, dtype="bf16"); n1.fc(n1.gap(n1.conv(n1.conv(0, cin, 3), cout, 1)), 10)
        n2 = N.Net("p", 16, 16, 10, dtype="bf16"); n2.fc(n2.gap(n2.conv(n2.conv(0, cin, 3), cout, 1, stride=2)), 10)
        n3 = N.Net("p", 16, 16, 10, dtype="bf16"); n3.fc(n3.gap(n3.conv(n3.conv(0, cin, 3), cout, 1, pre=True)), 10)
        assert ens.ens_spec_bytes(n1, 8)[0] == ens.ens_spec_bytes(n2, 8)[0]
        # (the pre-activation brings its own scale and shift per input channel)
        assert 0 <= ens.ens_spec_bytes(n3, 8)[0] + pointwise(cin, cout) - ens.ens_spec_bytes(n1, 8)[0] <= 2 * up(4 * cin) + 512
    plain, _ = ens.ens_spec_bytes(block(96, 256, 256, stride=2), 8)
    assert ens.ens_spec_bytes(block(96, 256, 256), 8)[0] == plain            # 96 channels in the middle
    w_tap, _ = ens.ens_spec_bytes(block(64, 256, 256, tap_t1=True), 8)
    w_tap2, _ = ens.ens_spec_bytes(block(64, 256, 256, stride=2, tap_t1=True), 8)
    assert w_tap == w_tap2                                                    # a second reader of t1
    assert ens.ens_spec_bytes(block(64, 256, 256, dtype="fp32"), 8)[0] == ens.ens_spec_bytes(block(64, 256, 256, stride=2, dtype="fp32"), 8)[0]
    assert ens.ens_spec_bytes(block(64, 48, 256), 8)[0] == ens.ens_spec_bytes(block(64, 48, 256, stride=2), 8)[0]   # input not in 32s
    assert pointwise(48, 64) == up(2 * 64 * 64)
