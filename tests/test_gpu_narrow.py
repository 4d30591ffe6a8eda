"""GPU parity of the narrow device layout: the repacking comes back byte for byte, and the GEMV on it agrees with the CPU oracle within 1e-4 of ||What[n,:]|| ||x|| and is
bitwise deterministic."""
import numpy as np
import pytest
import torch

from paper_2307_03738_amd import synth
from tests.util import dev, host, scaled_error

pytestmark = pytest.mark.gpu

TOL_FP32 = 1e-4


@pytest.fixture(scope="module")
def qg():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2307_03738_amd import binding
    binding.lib()
    return binding


def _announce(*what):
    print("[case]", *what, flush=True)


NARROW_CASES = [  # N, K, bits, group
    (16, 128, 4, 128),        # one tile of 16, one step: three of the four slices are padding
    (100, 512, 4, 128),       # one wave-step, ragged N
    (70, 640, 4, 128),        # five steps: the second wave-step holds a single real slice
    (300, 4096, 4, 128),      # eight wavefronts, one wave-step each (the 7B attention shape's K)
    (130, 11008, 4, 128),     # 86 steps: three wave-steps per wavefront, the last wave-step half real
    (200, 2048, 4, 32),       # four groups per step
    (90, 1024, 4, 16),        # eight groups per step
    (64, 1024, 4, 64),
    (1, 256, 4, 128),         # a single output
    (130, 5120, 3, 64),       # the 13B-shaped format
    (70, 768, 3, 256),
    (50, 1024, 3, 32),
    (33, 13824, 3, 64),
    (96, 2048, 2, 32),        # the 65B-shaped format
    (100, 768, 2, 256),
    (40, 512, 2, 16),         # sixteen groups per step
    (77, 22016, 2, 32),
    (20, 32768, 4, 128),      # the longest K the layout takes at 4 bits
]


@pytest.mark.parametrize("N,K,bits,group", NARROW_CASES)
def test_narrow_repack_comes_back_byte_for_byte(qg, N, K, bits, group):
    _announce("narrow repack", N, K, bits, group)
    W, _ = synth.small_case(N + K + bits, N, K, 0.02, True)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    blob = qg.qg_pack(q, s, z, bits, group)
    narrow = qg.qg_to_narrow(blob, N, K, bits, group)
    back = qg.qg_from_narrow(narrow, N, K, bits, group)
    torch.cuda.synchronize()
    assert narrow.numel() == qg.qg_packed_bytes(N, K, bits, group, qg.QG_LAYOUT_DEVICE_NARROW)
    assert np.array_equal(host(back), host(blob))
    # the scales move as they are: the same multiset of non-zero 32-bit words among the blob's
    # words that are no code words (a scale of the synthetic weights is no small integer, and a
    # word of zero-points or of codes that looks like one of them is not to be expected)
    sc = np.unique(host(s).view(np.uint32))
    sc = sc[sc != 0]
    for words in (host(narrow).view(np.uint32), host(blob).view(np.uint32)):
        assert np.array_equal(np.unique(words[np.isin(words, sc)]), sc)


@pytest.mark.parametrize("tpw", [0, 1, 2])        # the built-in choice; one and two tiles per wavefront
@pytest.mark.parametrize("N,K,bits,group", NARROW_CASES)
def test_gemv_narrow_matches_oracle(qg, oracle, N, K, bits, group, tpw):
    _announce("gemv narrow", N, K, bits, group, tpw)
    W, x = synth.small_case(N * 3 + K + group, N, K, 0.02, True)
    q0, s0, z0 = oracle.quantize(W, bits, group)
    y_ref, norms = oracle.matvec(q0, s0, z0, group, x), oracle.row_norms(q0, s0, z0, group)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    blob = qg.qg_pack(q, s, z, bits, group)
    narrow = qg.qg_to_narrow(blob, N, K, bits, group)
    y = torch.full((N + 64,), 7.0, dtype=torch.float32, device="cuda")          # canary behind y
    qg.qg_set_narrow_tuning(tpw)
    try:
        qg.qg_gemv_narrow(narrow, N, K, bits, group, dev(x), y[:N])
        y2 = qg.qg_gemv_narrow(narrow, N, K, bits, group, dev(x))
        torch.cuda.synchronize()
    finally:
        qg.qg_set_narrow_tuning(0)
    yh = host(y)
    assert np.all(yh[N:] == 7.0), "write past the end of y"
    assert np.array_equal(yh[:N], host(y2)), "not deterministic"
    assert scaled_error(yh[:N], y_ref, norms, x) <= TOL_FP32
    assert qg.qg_last_narrow_kernel().startswith(f"gemv_narrow<{bits}, ")


def test_gemv_narrow_formats_it_does_not_take(qg):
    # K that ends inside a step, groups of several steps, a group of one 4-bit cell, K beyond a workgroup
    for (N, K, bits, group) in [(64, 192, 4, 64), (64, 1024, 4, 256), (64, 1024, 4, 8), (16, 65536, 4, 128), (64, 1024, 3, 1024)]:
        assert qg.qg_packed_bytes(N, K, bits, group, qg.QG_LAYOUT_DEVICE_NARROW) == 0, (N, K, bits, group)
    blob = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    x = torch.zeros(1024, dtype=torch.float32, device="cuda")
    y = torch.zeros(64, dtype=torch.float32, device="cuda")
    assert qg.lib().qg_gemv_narrow(blob.data_ptr(), 64, 1024, 4, 256, x.data_ptr(), y.data_ptr(), None) == 3
    assert qg.lib().qg_to_narrow(blob.data_ptr(), 64, 1024, 4, 256, blob.data_ptr(), None) == 3


def test_gemv_narrow_non_finite_activations_reach_the_output(qg):
    _announce("gemv narrow non-finite")
    N, K, bits, group = 48, 1024, 4, 128
    W, x = synth.small_case(4242, N, K, 0.02, False)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    narrow = qg.qg_to_narrow(qg.qg_pack(q, s, z, bits, group), N, K, bits, group)
    for bad in (np.nan, np.inf, -np.inf):
        xb = x.copy()
        xb[517] = bad
        y = qg.qg_gemv_narrow(narrow, N, K, bits, group, dev(xb))
        torch.cuda.synchronize()
        assert not np.any(np.isfinite(host(y))), bad


def _hard_activations(K, kind, rng):
    """x vectors aimed at the fixed-point conversion of the kernel: values at the top of a step's
    range with both signs next to each other, one outlier among small values, tiny and zero steps."""
    top = np.float32(np.nextafter(np.float32(2.0), np.float32(0.0)))       # the largest mantissa
    if kind == "alternating top":
        x = np.where(np.arange(K) % 2 == 0, top, -top).astype(np.float32) * np.float32(1e4)
    elif kind == "negative top":
        x = np.full(K, -top, dtype=np.float32)
    elif kind == "pairs of opposite sign":
        x = (rng.standard_normal(K) * 3.0).astype(np.float32)
        x[1::2] = -16.0 * x[0::2]                                           # x_hi / 16 - x_lo = -2 x_lo
    elif kind == "outlier":
        x = (rng.standard_normal(K) * 1e-3).astype(np.float32)
        x[rng.integers(0, K, size=max(1, K // 512))] = np.float32(1e6)
    elif kind == "tiny and zero":
        x = (rng.standard_normal(K) * 1e-30).astype(np.float32)
        x[: K // 2] = 0.0
        x[K // 2 + 3] = np.float32(1e-42)                                   # a denormal
    else:
        raise ValueError(kind)
    return x


@pytest.mark.parametrize("kind", ["alternating top", "negative top", "pairs of opposite sign", "outlier", "tiny and zero"])
@pytest.mark.parametrize("N,K,bits,group", [(70, 4096, 4, 128), (33, 1024, 4, 32), (20, 512, 4, 16), (40, 2304, 3, 64),
                                            (50, 1536, 2, 32)])
def test_gemv_narrow_hard_activations(qg, oracle, N, K, bits, group, kind):
    _announce("gemv narrow hard x", N, K, bits, group, kind)
    rng = np.random.default_rng(N + K + len(kind))
    W, _ = synth.small_case(N + 5 * K + bits, N, K, 0.02, True)
    x = _hard_activations(K, kind, rng)
    q0, s0, z0 = oracle.quantize(W, bits, group)
    y_ref, norms = oracle.matvec(q0, s0, z0, group, x), oracle.row_norms(q0, s0, z0, group)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    narrow = qg.qg_to_narrow(qg.qg_pack(q, s, z, bits, group), N, K, bits, group)
    for tpw in (1, 2):
        qg.qg_set_narrow_tuning(tpw)
        try:
            y = qg.qg_gemv_narrow(narrow, N, K, bits, group, dev(x))
            torch.cuda.synchronize()
        finally:
            qg.qg_set_narrow_tuning(0)
        assert np.all(np.isfinite(host(y)))
        # the bound of the boundary, and the level the fixed point is built for (32-bit per step:
        # an error of a few 2^-24 of the step's largest |x| per weight)
        err = scaled_error(host(y), y_ref, norms, x)
        assert err <= TOL_FP32
        assert err <= 2e-6, (err, kind)


def test_gemv_narrow_replayed_from_a_graph(qg, oracle):
    # a serving loop captures the call once and replays it: every replay, with eager work and
    # synchronizations of the program in between, gives what the eager call gives on the same x
    _announce("gemv narrow in a graph")
    specs = [(300, 4096, 4, 128), (130, 1536, 3, 64), (96, 2048, 2, 32)]
    problems, refs = [], []
    for i, (N, K, bits, group) in enumerate(specs):
        W, x = synth.small_case(9100 + i, N, K, 0.02, True)
        q0, s0, z0 = oracle.quantize(W, bits, group)
        refs.append((q0, s0, z0, oracle.row_norms(q0, s0, z0, group)))
        q, s, z = qg.qg_quantize(dev(W), bits, group)
        problems.append(dict(packed=qg.qg_to_narrow(qg.qg_pack(q, s, z, bits, group), N, K, bits, group), N=N, K=K,
                             bits=bits, group=group, x=dev(x), y=torch.zeros(N, dtype=torch.float32, device="cuda")))
    launch = qg.GroupedGemvNarrow(problems)
    launch.launch()                                   # the kernels are loaded before the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        launch.launch()
    rng = np.random.default_rng(77)
    for replay in range(4):
        xs = [rng.standard_normal(p["K"]).astype(np.float32) * (replay + 1) for p in problems]
        for p, x in zip(problems, xs):
            p["x"].copy_(dev(x))
            p["y"].fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        replayed = [host(p["y"]).copy() for p in problems]
        launch.launch()
        torch.cuda.synchronize()
        for p, x, yr, (q0, s0, z0, norms) in zip(problems, xs, replayed, refs):
            assert np.array_equal(yr, host(p["y"])), (replay, p["N"], p["K"], p["bits"])
            assert scaled_error(yr, oracle.matvec(q0, s0, z0, p["group"], x), norms, x) <= TOL_FP32


def test_gemv_narrow_grouped_mixed_problems(qg, oracle):
    # one call, three kernel classes, K of different lengths inside a class, ragged N
    _announce("gemv narrow grouped")
    specs = [(300, 2048, 4, 128), (130, 11008, 4, 128), (70, 512, 4, 128), (100, 1024, 3, 64), (50, 1024, 2, 32),
             (16, 128, 4, 128), (90, 1536, 3, 64)]
    problems, refs = [], []
    for i, (N, K, bits, group) in enumerate(specs):
        W, x = synth.small_case(7000 + i, N, K, 0.02, True)
        q0, s0, z0 = oracle.quantize(W, bits, group)
        refs.append((oracle.matvec(q0, s0, z0, group, x), oracle.row_norms(q0, s0, z0, group), x))
        q, s, z = qg.qg_quantize(dev(W), bits, group)
        narrow = qg.qg_to_narrow(qg.qg_pack(q, s, z, bits, group), N, K, bits, group)
        problems.append(dict(packed=narrow, N=N, K=K, bits=bits, group=group, x=dev(x),
                             y=torch.full((N,), 7.0, dtype=torch.float32, device="cuda")))
    launch = qg.GroupedGemvNarrow(problems)
    for tpw in (1, 2):
        qg.qg_set_narrow_tuning(tpw)
        try:
            launch.launch()
            first = [host(p["y"]).copy() for p in problems]
            launch.launch()
            torch.cuda.synchronize()
        finally:
            qg.qg_set_narrow_tuning(0)
        for p, y1, (y_ref, norms, x) in zip(problems, first, refs):
            assert np.array_equal(host(p["y"]), y1), "not deterministic"
            assert scaled_error(y1, y_ref, norms, x) <= TOL_FP32
            p["y"].fill_(7.0)


@pytest.mark.parametrize("count", [12, 13, 14, 16])
def test_gemv_narrow_grouped_many_problems_of_one_format(qg, oracle, count):
    # one kernel launch with up to the maximum number of problems: the table of first workgroups is
    # searched in two parts, twelve entries in registers and the rest from the argument buffer
    _announce("gemv narrow grouped, one format", count)
    problems, refs = [], []
    for i in range(count):
        N, K, bits, group = 20 + 37 * i, 512 + 128 * (i % 5), 4, 128
        W, x = synth.small_case(4100 + i, N, K, 0.02, False)
        q0, s0, z0 = oracle.quantize(W, bits, group)
        refs.append((oracle.matvec(q0, s0, z0, group, x), oracle.row_norms(q0, s0, z0, group), x))
        q, s, z = qg.qg_quantize(dev(W), bits, group)
        problems.append(dict(packed=qg.qg_to_narrow(qg.qg_pack(q, s, z, bits, group), N, K, bits, group), N=N, K=K,
                             bits=bits, group=group, x=dev(x), y=torch.empty(N, dtype=torch.float32, device="cuda")))
    qg.GroupedGemvNarrow(problems).launch()
    torch.cuda.synchronize()
    for p, (y_ref, norms, x) in zip(problems, refs):
        assert scaled_error(host(p["y"]), y_ref, norms, x) <= TOL_FP32


@pytest.mark.parametrize("tpw", [1, 2])
@pytest.mark.parametrize("name", ["C2", "C3", "C4"])
def test_narrow_layer_set_full_size(qg, oracle, name, tpw):
    # the whole layer set in one grouped launch on the narrow layout, every output of every matrix
    # against the oracle; and against the wide layout's GEMV, which computes the same sums in another order
    cfg = synth.CONFIGS[name]
    _announce("narrow layer set", name)
    problems, wide, refs = [], [], []
    for i, (N, K) in enumerate(cfg.shapes):
        W, (x,) = synth.matrix(cfg, i)
        q0, s0, z0 = oracle.quantize(W, cfg.bits, cfg.group)
        refs.append((oracle.matvec(q0, s0, z0, cfg.group, x), oracle.row_norms(q0, s0, z0, cfg.group), x))
        q, s, z = qg.qg_quantize(dev(W), cfg.bits, cfg.group)
        del W, q0, s0, z0
        blob = qg.qg_pack(q, s, z, cfg.bits, cfg.group)
        del q, s, z
        xd = dev(x)
        problems.append(dict(packed=qg.qg_to_narrow(blob, N, K, cfg.bits, cfg.group), N=N, K=K, bits=cfg.bits,
                             group=cfg.group, x=xd, y=torch.empty(N, dtype=torch.float32, device="cuda")))
        wide.append(dict(packed=blob, N=N, K=K, bits=cfg.bits, group=cfg.group, x=xd,
                         y=torch.empty(N, dtype=torch.float32, device="cuda")))
    launch = qg.GroupedGemvNarrow(problems)
    qg.qg_set_narrow_tuning(tpw)
    try:
        launch.launch()
        first = [host(p["y"]).copy() for p in problems]
        launch.launch()
    finally:
        qg.qg_set_narrow_tuning(0)
    qg.qg_gemv_grouped(wide)
    torch.cuda.synchronize()
    worst = 0.0
    for p, pw, y1, (y_ref, norms, x) in zip(problems, wide, first, refs):
        assert np.array_equal(host(p["y"]), y1), "not deterministic"
        worst = max(worst, scaled_error(y1, y_ref, norms, x))
        assert scaled_error(y1, host(pw["y"]).astype(np.float64), norms, x) <= 1e-6
    print(f"[full] {name} narrow grouped launch, worst scaled error {worst:.3e}", flush=True)
    assert worst <= TOL_FP32, worst
