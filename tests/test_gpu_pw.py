"""Parity of prom_pw_conv (HIP, through the C ABI) against the CPU oracle: bit-exact."""
import numpy as np
import pytest

import oracle
from workloads import make_pw_layer, BASELINE_CONFIGS, CONFIG_SEED_BASE
from gpu_util import run_pw, oracle_pw, assert_same, dev, requant_dev, torch_cuda

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


def _cfg_layer(i):
    c = BASELINE_CONFIGS[i]
    return make_pw_layer(CONFIG_SEED_BASE + i, c["n"], c["h"], c["w"], c["cin"], c["cout"],
                         act_window=c["act_window"], with_residual=c["residual"])


@pytest.mark.parametrize("cfg", [0, 1, 2])
def test_baseline_configs_full_output(P, cfg):
    L = _cfg_layer(cfg)
    assert_same(run_pw(P, L), oracle_pw(oracle, L), f"config {cfg}")


EDGE_SHAPES = [
    # n, h, w, cin, cout  -- ragged pixel counts, channel counts off every tile size
    (1, 1, 1, 8, 4), (1, 3, 5, 16, 16), (1, 5, 13, 24, 20), (2, 7, 7, 40, 36),
    (1, 9, 9, 64, 144), (3, 5, 7, 72, 200), (1, 17, 3, 144, 24), (1, 11, 11, 200, 52),
    (1, 4, 4, 960, 160), (2, 6, 5, 328, 1280), (1, 31, 33, 32, 192), (1, 2, 2, 1024, 8),
    (1, 13, 7, 4096, 12),
]


@pytest.mark.parametrize("shape", EDGE_SHAPES)
@pytest.mark.parametrize("res", [False, True])
def test_edge_shapes_signed_inputs(P, shape, res):
    n, h, w, cin, cout = shape
    L = make_pw_layer(1000 + cin * 7 + cout, n, h, w, cin, cout, signed_x=True,
                      act_window=(-128, 127) if res else (-20, 90), with_residual=res,
                      shift_range=(3, 9))
    L.x.reshape(-1)[::37] = -128
    assert_same(run_pw(P, L), oracle_pw(oracle, L), f"shape {shape} res={res}")


GENERIC_SHAPES = [(1, 3, 3, 3, 5), (1, 5, 7, 17, 7), (2, 4, 4, 1, 1), (1, 6, 6, 24, 5),
                  (1, 6, 6, 13, 16), (1, 3, 11, 100, 33), (1, 2, 3, 4095, 6)]


@pytest.mark.parametrize("shape", GENERIC_SHAPES)
def test_generic_path_odd_channels(P, shape):
    n, h, w, cin, cout = shape
    L = make_pw_layer(2000 + cin * 3 + cout, n, h, w, cin, cout, signed_x=True,
                      act_window=(-128, 127), with_residual=True, shift_range=(0, 6))
    assert_same(run_pw(P, L), oracle_pw(oracle, L), f"generic shape {shape}")


def test_misaligned_pointers_take_the_generic_path(P):
    torch = torch_cuda()
    L = make_pw_layer(2100, 1, 7, 9, 32, 24, signed_x=True, act_window=(-128, 127), with_residual=True)
    want = oracle_pw(oracle, L)
    m = 63
    xbuf = torch.zeros(m * 32 + 8, dtype=torch.int8, device="cuda")
    ybuf = torch.zeros(m * 24 + 8, dtype=torch.int8, device="cuda")
    rbuf = torch.zeros(m * 24 + 8, dtype=torch.int8, device="cuda")
    for off in (1, 2, 3):
        xv = xbuf[off:off + m * 32].view(1, 7, 9, 32)
        xv.copy_(dev(L.x))
        yv = ybuf[off:off + m * 24].view(1, 7, 9, 24)
        rv = rbuf[off:off + m * 24].view(1, 7, 9, 24)
        rv.copy_(dev(L.residual))
        ybuf.fill_(77)
        P.prom_pw_conv(xv, dev(P.prom_pack_ternary(L.weight)), 24, requant_dev(P, L), rv, yv)
        torch.cuda.synchronize()
        assert_same(yv.cpu().numpy(), want, f"offset {off}")
        assert int(ybuf[off - 1]) == 77 and int(ybuf[off + m * 24]) == 77  # no write outside y


@pytest.mark.parametrize("nt", list(range(1, 11)))
def test_every_tile_plan(P, nt):
    """Every compiled (tiles per wave, pixel tiles) variant, on shapes whose channel count is
    not a multiple of the chunk, with both load widths (cin % 16 == 0 and cin % 16 == 8)."""
    for cin, cout in ((64, 192), (24, 144), (200, 100)):
        L = make_pw_layer(3000 + nt + cin, 2, 9, 13, cin, cout, signed_x=True,
                          act_window=(-100, 100), with_residual=(cin == 64))
        want = oracle_pw(oracle, L)
        for pt in (1, 2, 4):
            if pt > (4 if nt <= 2 else 2 if nt <= 6 else 1):
                continue
            for wgs in (0, 1, 3):
                plan = P.PwPlan(nt, pt, wgs)
                if cout % 16 != 0 and nt * 16 < cout:
                    # a channel count off the 16-byte piece size cannot be split into chunks
                    with pytest.raises(P.PromError) as e:
                        run_pw(P, L, plan=plan)
                    assert e.value.code == -1
                    continue
                assert_same(run_pw(P, L, plan=plan), want, f"nt={nt} pt={pt} wgs={wgs} cin={cin}")


@pytest.mark.parametrize("cw", [2, 3, 4])
def test_row_cooperative_plans(P, cw):
    """The row-cooperative kernel (2 or 4 wavefronts of a workgroup share a pixel group and write
    whole rows): every tile count, one and several k steps, ragged pixel counts down to a single
    pixel, few and many workgroups, with and without the skip connection."""
    for nt in range(1, 7):
        cout = 16 * nt * cw
        for (n, h, w, cin) in ((2, 9, 13, 32), (1, 7, 7, 160), (1, 1, 1, 64), (3, 5, 11, 16), (2, 6, 9, 24),
                               (1, 8, 5, 72)):
            L = make_pw_layer(5000 + 10 * nt + cw + cin, n, h, w, cin, cout, signed_x=True,
                              act_window=(-100, 100), with_residual=(cin == 32))
            want = oracle_pw(oracle, L)
            for wgs in (0, 1, 5):
                plan = P.PwPlan(nt, 0, wgs, cw)
                assert_same(run_pw(P, L, plan=plan), want, f"rows cw={cw} nt={nt} cin={cin} wgs={wgs}")
    # a row of several pieces (two pieces of 16*nt*cw channels)
    L = make_pw_layer(5900 + cw, 2, 6, 7, 48, 2 * 16 * 2 * cw, signed_x=True, with_residual=True,
                      act_window=(-128, 127))
    assert_same(run_pw(P, L, plan=P.PwPlan(2, 1, 0, cw)), oracle_pw(oracle, L), f"rows cw={cw} two pieces")
    # plans that cannot be realised
    L = make_pw_layer(5950, 1, 4, 4, 32, 96)
    for bad in (P.PwPlan(5, 0, 0, cw), P.PwPlan(7, 0, 0, cw), P.PwPlan(1, 2, 0, cw), P.PwPlan(1, 0, 0, 5)):
        with pytest.raises(P.PromError) as e:
            run_pw(P, L, plan=bad)
        assert e.value.code == -1
    L = make_pw_layer(5960, 1, 4, 4, 20, 16 * cw)  # cin % 8 != 0: not a fast-path shape
    with pytest.raises(P.PromError) as e:
        run_pw(P, L, plan=P.PwPlan(1, 0, 0, cw))
    assert e.value.code == -1


def test_library_picks_row_cooperative_kernel_for_wide_rows(P):
    """A 32->192 and a 64->384 layer (rows wider than one wavefront's chunk, whole row = 4
    wavefronts) take the row-cooperative kernel by default; results as the oracle's."""
    for cin, cout in ((32, 192), (64, 384), (32, 256), (24, 288)):
        q = P.prom_pw_plan_query(2, 28, 28, cin, cout)
        assert q["row_waves"] in (2, 3, 4) and 16 * q["tiles_per_wave"] * q["row_waves"] == cout, q
        L = make_pw_layer(5980 + cin, 2, 28, 28, cin, cout)
        assert_same(run_pw(P, L), oracle_pw(oracle, L), f"default plan {cin}->{cout}")
    assert P.prom_pw_plan_query(2, 28, 28, 16, 96)["row_waves"] == 0  # one chunk: plain kernel


def test_raw_accumulators(P):
    torch = torch_cuda()
    for cin, cout in ((64, 384), (24, 144), (17, 5), (960, 160)):
        L = make_pw_layer(4000 + cin, 1, 7, 9, cin, cout, signed_x=True)
        acc = P.prom_pw_accum_i32(dev(L.x), dev(P.prom_pack_ternary(L.weight)), cout)
        torch.cuda.synchronize()
        assert_same(acc.cpu().numpy(), oracle.pw_accum(L.x, L.weight), f"accum {cin}x{cout}")


def test_closed_forms_on_gpu(P):
    """All-zero weights give the requantised bias; all +1 give row sums."""
    L = make_pw_layer(4100, 1, 8, 8, 48, 32, signed_x=True, act_window=(-128, 127))
    L.weight[:] = 0
    y = run_pw(P, L)
    assert_same(y, oracle_pw(oracle, L), "zero weights")
    assert (y == y[0, 0, 0]).all()
    L.weight[:] = 1
    assert_same(run_pw(P, L), oracle_pw(oracle, L), "all +1 weights")
    L.weight[:] = -1
    assert_same(run_pw(P, L), oracle_pw(oracle, L), "all -1 weights")


CRAFTED = [(1 << 30, 8), (1 << 30, 0), ((1 << 31) - 1, 14), ((1 << 30) + 1, 9),
           (0x5A5A5A5B, 11), (0x7FFFFFFF, 0), (0x40000000, 31), (0x6DB6DB6E, 13), (1, 0), (3, 31)]


def test_epilogue_sweep_every_s_and_ties(P):
    """Identity-like weights turn the layer into a pure epilogue test: s = x + bias[c] sweeps
    every integer in [-4224, 4223] (and a wide range scaled by 2^k) for crafted (mult, shift),
    including exact .5 ties."""
    x = np.tile(np.arange(-128, 128, dtype=np.int16).astype(np.int8).reshape(256, 1), (1, 8))
    x = np.ascontiguousarray(x).reshape(1, 16, 16, 8)
    cout = 33 * len(CRAFTED)
    w = np.zeros((cout, 8), dtype=np.int8)
    w[:, 0] = 1
    bias = np.zeros(cout, np.int32); mult = np.zeros(cout, np.int32); shift = np.zeros(cout, np.int32)
    for i, (m, s) in enumerate(CRAFTED):
        for b in range(33):
            c = i * 33 + b
            bias[c] = -4096 + 256 * b
            mult[c], shift[c] = m, s
    L = make_pw_layer(1, 1, 16, 16, 8, cout)
    L.x, L.weight, L.bias, L.mult, L.shift = x, w, bias, mult, shift
    for window in ((-128, 127), (0, 127), (-7, 7)):
        assert_same(run_pw(P, L, window=window), oracle_pw(oracle, L, window=window), f"sweep {window}")
    # large |s|: biases up to 2^29 in magnitude (the documented bound is |acc + bias| < 2^30)
    L.bias = (bias.astype(np.int64) * (1 << 17)).clip(-(1 << 29), 1 << 29).astype(np.int32)
    assert_same(run_pw(P, L, window=(-128, 127)), oracle_pw(oracle, L, window=(-128, 127)), "large s")


def test_residual_may_alias_output(P):
    torch = torch_cuda()
    L = make_pw_layer(4200, 2, 7, 7, 96, 40, act_window=(-128, 127), with_residual=True)
    want = oracle_pw(oracle, L)
    y = dev(L.residual).clone()
    P.prom_pw_conv(dev(L.x), dev(P.prom_pack_ternary(L.weight)), 40, requant_dev(P, L), y, y)
    torch.cuda.synchronize()
    assert_same(y.cpu().numpy(), want, "in-place residual")


def test_zero_fraction_variants(P):
    """Weight zero fractions from the paper's initialisation (31 %) to its trained maximum (55 %)."""
    for pz in (0.0, 0.31, 0.55, 1.0):
        L = make_pw_layer(4300, 1, 14, 14, 64, 384, p_zero=pz)
        assert_same(run_pw(P, L), oracle_pw(oracle, L), f"p_zero={pz}")


ADDSUB_SHAPES = [(1, 14, 14, 64, 384), (2, 28, 28, 24, 144), (1, 9, 13, 144, 24), (3, 7, 7, 16, 96),
                 (1, 5, 11, 256, 40), (1, 3, 3, 4, 4), (2, 14, 14, 192, 64), (1, 10, 10, 96, 576)]


@pytest.mark.parametrize("shape", ADDSUB_SHAPES)
@pytest.mark.parametrize("res", [False, True])
def test_addsub_design_matches_oracle(P, shape, res):
    """The vector-ALU add/subtract design (kept for the A/B measurement) is bit-exact too."""
    torch = torch_cuda()
    n, h, w, cin, cout = shape
    L = make_pw_layer(7000 + cin + cout, n, h, w, cin, cout, signed_x=True,
                      act_window=(-128, 127) if res else (0, 127), with_residual=res, shift_range=(2, 9))
    L.x.reshape(-1)[::41] = -128
    y = P.prom_pw_conv_addsub(dev(L.x), dev(P.prom_pack_ternary(L.weight)), cout, requant_dev(P, L),
                              dev(L.residual) if res else None)
    torch.cuda.synchronize()
    assert_same(y.cpu().numpy(), oracle_pw(oracle, L), f"addsub {shape} res={res}")


def test_sequence_batches_independent_layers_and_respects_dependencies(P):
    """prom_pw_conv_sequence puts consecutive small independent layers into one launch; its
    results must be those of running the layers one after the other, also when a layer reads
    what an earlier one wrote, writes what an earlier one read, or adds its own output buffer."""
    torch = torch_cuda()
    shapes = [(64, 64), (64, 96), (96, 160), (160, 64), (64, 384), (384, 64), (64, 32), (32, 192), (24, 144)]
    n, h, w = 3, 7, 9
    Ls = [make_pw_layer(8000 + i, n, h, w, ci, co, signed_x=True, act_window=(-128, 127), shift_range=(3, 8))
          for i, (ci, co) in enumerate(shapes)]
    # oracle: a chain where layer i+1 reads layer i's output when the channel counts match
    want, x_in = [], []
    prev = None
    for i, L in enumerate(Ls):
        x = prev if (prev is not None and prev.shape[-1] == L.cin) else L.x
        x_in.append(x)
        prev = oracle.pw_conv(x, L.weight, L.bias, L.mult, L.shift, -128, 127)
        want.append(prev)
    # device: same wiring, buffers shared exactly as in the chain
    ys = [torch.empty((n, h, w, L.cout), dtype=torch.int8, device="cuda") for L in Ls]
    layers = []
    for i, L in enumerate(Ls):
        chained = i > 0 and Ls[i - 1].cout == L.cin
        xd = ys[i - 1] if chained else dev(L.x)
        layers.append((xd, dev(P.prom_pack_ternary(L.weight)), L.cout, requant_dev(P, L, (-128, 127)), None, ys[i]))
    P.PwSequence(layers).run()
    torch.cuda.synchronize()
    for i, (y, wnt) in enumerate(zip(ys, want)):
        assert_same(y.cpu().numpy(), wnt, f"sequence layer {i} {shapes[i]}")
    # fully independent copies of the same layers (all batchable ones in one launch) + in-place residual
    ys2 = [dev(np.ascontiguousarray(w_)) for w_ in want]  # used as residual and output at once
    layers2 = [(dev(x_in[i]), dev(P.prom_pack_ternary(L.weight)), L.cout, requant_dev(P, L, (-128, 127)), ys2[i], ys2[i])
               for i, L in enumerate(Ls)]
    P.PwSequence(layers2).run()
    torch.cuda.synchronize()
    for i, L in enumerate(Ls):
        wnt = oracle.pw_conv(x_in[i], L.weight, L.bias, L.mult, L.shift, -128, 127, want[i])
        assert_same(ys2[i].cpu().numpy(), wnt, f"independent layer {i} with in-place residual")


def test_sequence_of_more_independent_layers_than_two_launches_hold(P):
    """75 independent small layers of mixed sizes in one call (a shared launch holds 32, the
    library lets 64 wait and deals them out by size), then one layer that reads the first
    layer's output: every output against the oracle."""
    torch = torch_cuda()
    shapes = [(16 * (1 + i % 6), 16 * (1 + (i * 5) % 7)) for i in range(75)]
    Ls = [make_pw_layer(8300 + i, 1 + i % 3, 5 + i % 4, 7, ci, co, signed_x=True, act_window=(-128, 127),
                        shift_range=(3, 8)) for i, (ci, co) in enumerate(shapes)]
    ys = [torch.empty((L.x.shape[0], L.x.shape[1], L.x.shape[2], L.cout), dtype=torch.int8, device="cuda") for L in Ls]
    layers = [(dev(L.x), dev(P.prom_pack_ternary(L.weight)), L.cout, requant_dev(P, L, (-128, 127)), None, y)
              for L, y in zip(Ls, ys)]
    last = make_pw_layer(8399, Ls[0].x.shape[0], Ls[0].x.shape[1], 7, Ls[0].cout, 48, signed_x=True,
                         act_window=(-128, 127), shift_range=(3, 8))
    y_last = torch.empty((*Ls[0].x.shape[:3], 48), dtype=torch.int8, device="cuda")
    layers.append((ys[0], dev(P.prom_pack_ternary(last.weight)), 48, requant_dev(P, last, (-128, 127)), None, y_last))
    P.PwSequence(layers).run()
    torch.cuda.synchronize()
    want0 = None
    for i, (L, y) in enumerate(zip(Ls, ys)):
        want = oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, -128, 127)
        if i == 0:
            want0 = want
        assert_same(y.cpu().numpy(), want, f"independent layer {i} {shapes[i]}")
    assert_same(y_last.cpu().numpy(),
                oracle.pw_conv(want0, last.weight, last.bias, last.mult, last.shift, -128, 127), "dependent last layer")


def test_pixel_tile_plans_agree_on_a_full_size_layer(P):
    """Regression: with two or four pixel tiles per step the 16-byte output stores of one step
    follow each other closely, and the registers of a store were once reused before the store had
    read them (a few wrong dwords per launch, only under full load).  Every output of a
    full-size 96->24 layer, for every pixel-tile count, on several runs, against the oracle."""
    torch = torch_cuda()
    L = make_pw_layer(4242, 128, 56, 56, 96, 24)
    x, wp, rq = dev(L.x), dev(P.prom_pack_ternary(L.weight)), requant_dev(P, L)
    want = dev(oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, L.act_min, L.act_max))
    for plan in (None, P.PwPlan(2, 1, 0), P.PwPlan(2, 2, 0), P.PwPlan(2, 4, 0)):
        for run in range(6):
            y = torch.full((128, 56, 56, 24), -99, dtype=torch.int8, device="cuda")
            P.prom_pw_conv_ex(x, wp, 24, rq, None, y, plan)
            torch.cuda.synchronize()
            bad = int((y != want).sum())
            assert bad == 0, f"plan {plan}, run {run}: {bad} outputs differ"


def test_sequence_puts_large_layers_into_one_launch(P):
    """Large independent layers whose plan the large-layer batch kernel carries (the head of
    MobileNetV2 at batch 64: 32->16, 16->96, 24->144 and 96->24) go through prom_pw_conv_sequence
    together with small ones; every output against the oracle, and a second call where the layers
    depend on each other (the output of one is the input of the next), which must not be batched."""
    torch = torch_cuda()
    shapes = [(112, 32, 16), (112, 16, 96), (56, 24, 144), (56, 96, 24), (14, 64, 384), (7, 160, 960)]
    n = 64
    classes = [P.prom_pw_batch_class(n, hw, hw, cin, cout) for hw, cin, cout in shapes]
    assert classes[:4] == [2, 2, 2, 2] and classes[4:] == [1, 1], classes
    layers, wants = [], []
    for i, (hw, cin, cout) in enumerate(shapes):
        L = make_pw_layer(9100 + i, n, hw, hw, cin, cout, signed_x=True, act_window=(-128, 127))
        y = torch.full((n, hw, hw, cout), -99, dtype=torch.int8, device="cuda")
        layers.append((dev(L.x), dev(P.prom_pack_ternary(L.weight)), cout, requant_dev(P, L), None, y))
        wants.append(dev(oracle_pw(oracle, L)))
    for run in range(3):
        for l in layers:
            l[5].fill_(-99)
        P.PwSequence(layers).run()
        torch.cuda.synchronize()
        for (hw, cin, cout), l, want in zip(shapes, layers, wants):
            assert int((l[5] != want).sum()) == 0, f"run {run}: {cin}->{cout} @ {hw}"
    # a chain 32 -> 16 -> 96 at 112x112: the second layer reads what the first writes
    n = 48
    A = make_pw_layer(9200, n, 112, 112, 32, 16, signed_x=True, act_window=(-128, 127), shift_range=(2, 3))
    Bq = make_pw_layer(9201, n, 112, 112, 16, 96, act_window=(-128, 127), shift_range=(1, 2), make_x=False)
    mid = torch.full((n, 112, 112, 16), -99, dtype=torch.int8, device="cuda")
    out = torch.full((n, 112, 112, 96), -99, dtype=torch.int8, device="cuda")
    P.PwSequence([(dev(A.x), dev(P.prom_pack_ternary(A.weight)), 16, requant_dev(P, A), None, mid),
                  (mid, dev(P.prom_pack_ternary(Bq.weight)), 96, requant_dev(P, Bq), None, out)]).run()
    torch.cuda.synchronize()
    m = oracle.pw_conv(A.x, A.weight, A.bias, A.mult, A.shift, -128, 127)
    want = oracle.pw_conv(m, Bq.weight, Bq.bias, Bq.mult, Bq.shift, -128, 127)
    assert_same(out.cpu().numpy(), want, "dependent large layers")


def test_sequence_expansion_layers_keep_activations_in_registers(P):
    """Layers with at most 192 input channels and a multiple of 64 output channels, no residual,
    take a body of their own inside the shared launch (activations of a pixel group in registers,
    output channels walked in sub-chunks of 64, in parts when their fragments do not fit LDS
    together).  One, two and three k steps with and without a ragged last step, part counts 1..5
    with an uneven last part, pixel counts that leave ragged units and tiles, channels with shift
    0 (general form of the requantisation) in one layer only; buffers pre-filled so that a
    missed or misplaced store shows; neighbours in the launch that take the streaming body."""
    torch = torch_cuda()
    cases = [  # n, h, w, cin, cout, shift_range
        (3, 7, 9, 32, 192, (3, 8)), (2, 14, 14, 64, 384, (3, 8)), (5, 5, 5, 16, 64 * 9, (2, 6)),
        (1, 31, 3, 48, 64 * 10, (0, 4)), (3, 14, 14, 96, 576, (3, 8)), (2, 9, 11, 128, 64 * 11, (1, 7)),
        (4, 7, 7, 160, 960, (3, 8)), (1, 13, 13, 192, 64 * 7, (0, 3)), (2, 6, 7, 144, 128, (2, 9)),
        (1, 1, 1, 64, 128, (3, 8)), (1, 1, 17, 80, 256, (3, 8)),
        (2, 7, 7, 320, 1280, (3, 8)), (3, 7, 9, 384, 64, (3, 8)), (3, 7, 9, 64, 96, (3, 8)),  # streaming body
    ]
    layers, wants = [], []
    for i, (n, h, w, cin, cout, sr) in enumerate(cases):
        L = make_pw_layer(9500 + i, n, h, w, cin, cout, signed_x=True, act_window=(-128, 127), shift_range=sr)
        y = torch.full((n, h, w, cout), -99, dtype=torch.int8, device="cuda")
        layers.append((dev(L.x), dev(P.prom_pack_ternary(L.weight)), cout, requant_dev(P, L), None, y))
        wants.append(oracle_pw(oracle, L))
    seq = P.PwSequence(layers)
    for run in range(2):
        for l in layers:
            l[5].fill_(-99)
        seq.run()
        torch.cuda.synchronize()
        for c, l, want in zip(cases, layers, wants):
            assert_same(l[5].cpu().numpy(), want, f"run {run}: case {c}")


def test_sequence_large_wide_row_layers_ragged_pixel_count(P):
    """24 -> 144 at high resolution inside the launch of large layers runs in the body where one
    wavefront assembles whole output rows of a 64-pixel unit; here with pixel counts that leave a
    ragged last unit and a ragged last 16-pixel tile, a second such layer with 48 output channels
    per pixel more, and a 16 -> 96 neighbour; outputs pre-filled, every byte compared."""
    torch = torch_cuda()
    shapes = [(65, 56, 55, 24, 144), (33, 111, 56, 24, 192), (64, 112, 112, 16, 96), (37, 113, 57, 24, 144)]
    classes = [P.prom_pw_batch_class(n, h, w, cin, cout) for n, h, w, cin, cout in shapes]
    assert classes == [2, 2, 2, 2], classes
    layers, wants = [], []
    for i, (n, h, w, cin, cout) in enumerate(shapes):
        assert (n * h * w) % 64 != 0 or cin == 16
        L = make_pw_layer(9700 + i, n, h, w, cin, cout, signed_x=True, act_window=(-128, 127), shift_range=(0, 6) if i == 3 else (2, 7))
        y = torch.full((n, h, w, cout), -99, dtype=torch.int8, device="cuda")
        layers.append((dev(L.x), dev(P.prom_pack_ternary(L.weight)), cout, requant_dev(P, L), None, y))
        wants.append(dev(oracle_pw(oracle, L)))
    seq = P.PwSequence(layers)
    for run in range(2):
        for l in layers:
            l[5].fill_(-99)
        seq.run()
        torch.cuda.synchronize()
        for sh, l, want in zip(shapes, layers, wants):
            assert int((l[5] != want).sum()) == 0, f"run {run}: {sh}"


def test_sequence_deep_projection_layers_keep_weights_in_registers(P):
    """Layers with 6, 9 or 15 k steps (384, 576, 960 input channels and ragged variants) inside the
    shared launch of small layers run the body that holds the weights in registers and passes the
    activations through LDS.  Group counts 1 and 2 with a ragged last group, channel tiles that
    leave wavefronts idle, pixel counts with a ragged last 16-pixel tile and fewer tiles than a
    prefetch round, enough pixels for several workgroups and rounds, residual (also in place),
    channels with shift 0, cin not a multiple of 64; outputs pre-filled, every byte compared."""
    torch = torch_cuda()
    cases = [  # n, h, w, cin, cout, shift_range, residual
        (3, 7, 9, 384, 96, (3, 8), False), (3, 7, 9, 576, 96, (3, 8), True), (2, 7, 7, 576, 160, (3, 8), False),
        (4, 7, 7, 960, 160, (3, 8), True), (5, 7, 7, 960, 320, (2, 9), False), (1, 1, 1, 960, 320, (3, 8), False),
        (1, 3, 5, 576, 112, (0, 5), True), (2, 5, 3, 912, 208, (3, 8), False), (1, 9, 9, 336, 128, (0, 3), False),
        (64, 14, 14, 576, 96, (3, 8), False), (40, 14, 14, 384, 96, (3, 8), True), (96, 7, 7, 960, 320, (3, 8), True),
        (3, 7, 9, 64, 96, (3, 8), False), (3, 7, 9, 32, 192, (3, 8), False),  # neighbours with other bodies
    ]
    layers, wants = [], []
    for i, (n, h, w, cin, cout, sr, res) in enumerate(cases):
        L = make_pw_layer(9800 + i, n, h, w, cin, cout, signed_x=True, act_window=(-128, 127), shift_range=sr,
                          with_residual=res)
        y = torch.full((n, h, w, cout), -99, dtype=torch.int8, device="cuda")
        r = dev(L.residual) if res else None
        layers.append((dev(L.x), dev(P.prom_pack_ternary(L.weight)), cout, requant_dev(P, L), r, y))
        wants.append(oracle_pw(oracle, L, residual=res))
    seq = P.PwSequence(layers)
    for run in range(2):
        for l in layers:
            l[5].fill_(-99)
        seq.run()
        torch.cuda.synchronize()
        for c, l, want in zip(cases, layers, wants):
            assert_same(l[5].cpu().numpy(), want, f"run {run}: case {c}")
    # the residual read from the output buffer itself
    inplace = []
    for c, l, (n, h, w, cin, cout, sr, res) in zip(cases, layers, cases):
        if res:
            yb = l[4].clone()
            inplace.append((c, (l[0], l[1], l[2], l[3], yb, yb)))
    P.PwSequence([l for _c, l in inplace]).run()
    torch.cuda.synchronize()
    for (c, l) in inplace:
        i = cases.index(c)
        assert_same(l[5].cpu().numpy(), wants[i], f"in-place residual: case {c}")
