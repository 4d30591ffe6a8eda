"""GPU parity: the HIP library, called through its C-ABI, against the CPU oracle on the same
seeded inputs.  Quantize, pack and unpack must agree bit for bit; products must agree within
1e-4 of ||What[n,:]|| ||x|| (fp32 path)."""
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


# ------------------------------------------------------------------ quantize (bit-exact)

QUANT_CASES = [  # N, K, bits, group, std, outliers
    (512, 512, 4, 64, 0.02, False),       # configuration 1
    (200, 768, 4, 128, 0.02, True),
    (130, 640, 3, 64, 0.02, False),
    (77, 512, 2, 32, 0.015, False),
    (64, 256, 2, 16, 0.02, False),
    (33, 384, 3, 32, 0.02, True),
    (16, 1024, 4, 1024, 0.02, True),      # one group per output (full column)
    (9, 96, 4, 8, 0.02, False),
    (5, 120, 4, 24, 1.0, False),
    (7, 8192, 4, 4096, 0.02, True),       # the largest group held in registers
    (3, 16384, 2, 8192, 0.02, False),     # larger: the looping kernel
    (37, 1536, 3, 512, 0.02, True),
    (1003, 256, 4, 256, 0.02, False),     # a last workgroup with idle teams
]


@pytest.mark.parametrize("N,K,bits,group,std,outliers", QUANT_CASES)
def test_quantize_bit_exact(qg, oracle, N, K, bits, group, std, outliers):
    _announce("quantize", N, K, bits, group)
    W, _ = synth.small_case(N * 7 + K, N, K, std, outliers)
    q0, s0, z0 = oracle.quantize(W, bits, group)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    assert np.array_equal(host(q), q0)
    assert np.array_equal(host(s).view(np.uint32), s0.view(np.uint32))
    assert np.array_equal(host(z), z0)


def test_quantize_special_values_bit_exact(qg, oracle):
    _announce("quantize special values")
    G = 16
    rows = [
        np.array([0.0, 15.0, 0.5, 1.5, 2.5, 3.5, 6.5, 13.5] + [0.0] * 8),      # exact ties, s = 1
        np.array([-1.0, 14.0, 0.5, 1.5, 2.5, -0.5] + [0.0] * 10),               # ties with odd zero
        np.zeros(G),                                                            # range 0
        np.linspace(0.25, 1.0, G),                                              # all positive
        -np.linspace(0.25, 1.0, G),                                             # all negative
        np.full(G, 1e-41),                                                      # denormals
        np.array([-0.0] * 8 + [3e-39] * 8),
        np.array([1e30, -1e30] + [1.0] * 14),                                   # huge range
    ]
    W = np.stack(rows).astype(np.float32)
    for bits in (2, 3, 4):
        q0, s0, z0 = oracle.quantize(W, bits, G)
        q, s, z = qg.qg_quantize(dev(W), bits, G)
        assert np.array_equal(host(q), q0), bits
        assert np.array_equal(host(s).view(np.uint32), s0.view(np.uint32)), bits
        assert np.array_equal(host(z), z0), bits


# ------------------------------------------------------------------ pack / unpack (bit-exact)

PACK_CASES = [(512, 512, 4, 64), (200, 768, 4, 128), (130, 640, 3, 64), (77, 512, 2, 32),
              (64, 256, 2, 16), (33, 384, 3, 32), (1, 96, 3, 96), (65, 160, 4, 32), (3, 64, 2, 64),
              # rows that are not multiples of 16 bytes; more than one block of columns per tile
              (70, 72, 4, 24), (9, 40, 4, 8), (129, 1160, 4, 8), (131, 1056, 3, 32), (67, 2064, 2, 16)]


@pytest.mark.parametrize("N,K,bits,group", PACK_CASES)
def test_canonical_pack_matches_oracle_words(qg, oracle, N, K, bits, group):
    _announce("canonical pack", N, K, bits, group)
    rng = np.random.default_rng(N + K + bits)
    q = rng.integers(0, 1 << bits, (N, K), dtype=np.uint8)
    z = rng.integers(0, 1 << bits, (N, K // group), dtype=np.uint8)
    s = rng.standard_normal((N, K // group)).astype(np.float32)
    blob = host(qg.qg_pack(dev(q), dev(s), dev(z), bits, group, qg.QG_LAYOUT_CANONICAL))
    P, St, Zp = oracle.pack_codes(q, bits), oracle.transpose_scales(s), oracle.pack_zeros(z, bits)
    ref = np.concatenate([P.ravel().view(np.uint8), St.ravel().view(np.uint8), Zp.ravel().view(np.uint8)])
    assert blob.size == ref.size == qg.qg_packed_bytes(N, K, bits, group, qg.QG_LAYOUT_CANONICAL)
    assert np.array_equal(blob, ref)
    # and back, from the oracle's words
    q2, s2, z2 = qg.qg_unpack(dev(ref), N, K, bits, group, qg.QG_LAYOUT_CANONICAL)
    assert np.array_equal(host(q2), q) and np.array_equal(host(z2), z)
    assert np.array_equal(host(s2).view(np.uint32), s.view(np.uint32))


@pytest.mark.parametrize("N,K,bits,group", PACK_CASES)
def test_device_pack_unpack_identity(qg, N, K, bits, group):
    _announce("device pack round trip", N, K, bits, group)
    rng = np.random.default_rng(N * 3 + K + bits)
    q = rng.integers(0, 1 << bits, (N, K), dtype=np.uint8)
    z = rng.integers(0, 1 << bits, (N, K // group), dtype=np.uint8)
    s = rng.standard_normal((N, K // group)).astype(np.float32)
    blob = qg.qg_pack(dev(q), dev(s), dev(z), bits, group, qg.QG_LAYOUT_DEVICE)
    q2, s2, z2 = qg.qg_unpack(blob, N, K, bits, group, qg.QG_LAYOUT_DEVICE)
    assert np.array_equal(host(q2), q) and np.array_equal(host(z2), z)
    assert np.array_equal(host(s2).view(np.uint32), s.view(np.uint32))


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_pack_from_unaligned_arrays(qg, oracle, bits):
    """Codes and zero-points that do not start on a 16-byte boundary take the byte-wise path."""
    N, K, group = 75, 512, 32
    _announce("unaligned pack", N, K, bits, group)
    rng = np.random.default_rng(40 + bits)
    q = rng.integers(0, 1 << bits, (N, K), dtype=np.uint8)
    z = rng.integers(0, 1 << bits, (N, K // group), dtype=np.uint8)
    s = rng.standard_normal((N, K // group)).astype(np.float32)
    qd = torch.empty(N * K + 16, dtype=torch.uint8, device="cuda")[3:3 + N * K].view(N, K)
    zd = torch.empty(z.size + 16, dtype=torch.uint8, device="cuda")[5:5 + z.size].view(N, K // group)
    qd.copy_(dev(q)); zd.copy_(dev(z))
    assert qd.data_ptr() % 16 and zd.data_ptr() % 16
    for layout in (qg.QG_LAYOUT_CANONICAL, qg.QG_LAYOUT_DEVICE):
        blob = qg.qg_pack(qd, dev(s), zd, bits, group, layout)
        assert torch.equal(blob, qg.qg_pack(dev(q), dev(s), dev(z), bits, group, layout))
        nbytes = qg.qg_packed_bytes(N, K, bits, group, layout)
        lib = qg.lib()
        q2 = torch.zeros(N * K + 16, dtype=torch.uint8, device="cuda")
        z2 = torch.zeros(z.size + 16, dtype=torch.uint8, device="cuda")
        s2 = torch.empty_like(dev(s))
        rc = lib.qg_unpack(blob.data_ptr(), N, K, bits, group, layout, q2.data_ptr() + 3, s2.data_ptr(),
                           z2.data_ptr() + 5, torch.cuda.current_stream().cuda_stream)
        assert rc == 0 and blob.numel() == nbytes
        torch.cuda.synchronize()
        assert np.array_equal(host(q2)[3:3 + N * K].reshape(N, K), q)
        assert np.array_equal(host(z2)[5:5 + z.size].reshape(N, -1), z)
        assert not host(q2)[:3].any() and not host(q2)[3 + N * K:].any()      # nothing written outside
        assert not host(z2)[:5].any() and not host(z2)[5 + z.size:].any()
        assert np.array_equal(host(s2).view(np.uint32), s.view(np.uint32))


# ------------------------------------------------------------------ GEMV (tolerance)

def _gemv_case(qg, oracle, W, x, bits, group, tuning=(0, 0, 0)):
    N, K = W.shape
    q0, s0, z0 = oracle.quantize(W, bits, group)
    y_ref = oracle.matvec(q0, s0, z0, group, x)
    norms = oracle.row_norms(q0, s0, z0, group)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    assert np.array_equal(host(q), q0) and np.array_equal(host(z), z0)
    assert np.array_equal(host(s).view(np.uint32), s0.view(np.uint32))
    blob = qg.qg_pack(q, s, z, bits, group, qg.QG_LAYOUT_DEVICE)
    qg.qg_set_gemv_tuning(*tuning)
    try:
        ws = qg.new_workspace(qg.qg_workspace_bytes(N, K, bits, group, 1))
        y = torch.full((N + 64,), 7.0, dtype=torch.float32, device="cuda")   # canary behind y
        qg.qg_gemv(blob, N, K, bits, group, dev(x), y[:N], ws)
        y2 = torch.empty(N, dtype=torch.float32, device="cuda")
        qg.qg_gemv(blob, N, K, bits, group, dev(x), y2, ws)                    # workspace reuse
        torch.cuda.synchronize()
    finally:
        qg.qg_set_gemv_tuning(0, 0, 0)
    yh = host(y)
    assert np.all(yh[N:] == 7.0), "write past the end of y"
    assert np.array_equal(yh[:N], host(y2)), "not deterministic / workspace not left clean"
    assert np.all(host(ws) == 0xFF), "workspace not left in its prepared state"
    return scaled_error(yh[:N], y_ref, norms, x)


GEMV_CASES = [  # N, K, bits, group   -- (kernel flavour)
    (512, 512, 4, 64),        # configuration 1, static groups
    (200, 1024, 4, 128),      # ragged N (3 tiles + 8)
    (130, 512, 4, 32),
    (70, 256, 4, 16),
    (64, 128, 4, 8),
    (257, 1024, 2, 32),
    (130, 512, 2, 16),
    (96, 768, 2, 64),
    (200, 1024, 2, 256),
    (130, 1536, 3, 64),
    (77, 512, 3, 32),
    (64, 1024, 3, 128),
    (200, 512, 3, 256),
    (150, 1024, 4, 256),      # group = two steps (runtime-group kernel)
    (100, 2048, 4, 2048),     # one group per output, eq. (1)
    (100, 1024, 2, 512),
    (66, 1536, 3, 768),
    (130, 11008, 4, 11008),   # full column, K long enough to be cut over wavefronts and workgroups
    (70, 5120, 3, 5120),
    (70, 8192, 2, 8192),
    (200, 2304, 4, 768),      # three groups of six steps: wavefront ranges end inside groups
    (90, 480, 4, 24),         # generic kernel: group not a power of two
    (90, 416, 4, 32),         # generic kernel: K not a whole number of steps
    (50, 288, 3, 96),
    (40, 336, 2, 48),
    (1, 128, 4, 128),         # a single output
]


@pytest.mark.parametrize("kernel", [0, 1, 2])    # the built-in choice / the vector ALU / the 32 x 32 x 16 matrix instruction
@pytest.mark.parametrize("N,K,bits,group", GEMV_CASES)
def test_gemv_matches_oracle(qg, oracle, N, K, bits, group, kernel):
    _announce("gemv", N, K, bits, group, kernel)
    W, x = synth.small_case(N + 3 * K + bits, N, K, 0.02, True)
    err = _gemv_case(qg, oracle, W, x, bits, group, (0, 0, kernel))
    assert err <= TOL_FP32, err


@pytest.mark.parametrize("bits,group", [(4, 16), (4, 32), (4, 64), (4, 128), (2, 32), (2, 64), (2, 128), (2, 256),
                                        (3, 64), (3, 128), (3, 256),
                                        # groups of whole steps: the accumulators run across steps
                                        (2, 512), (2, 2048), (3, 512), (3, 1024), (3, 2048), (4, 256), (4, 2048)])
@pytest.mark.parametrize("kernel", [2, 3, 4])
def test_gemv_matrix_core_kernel_every_group_size(qg, oracle, bits, group, kernel):
    # x with a wide range of magnitudes and both signs: its split into three bf16 parts must be exact
    # (kernel 2: 32x32x16 matrix instruction, 3: 4x4x4 on bf16, 4: 4x4x4 on int8 with x in 32-bit fixed point)
    _announce("gemv matrix cores", bits, group, kernel)
    N, K = 200, 2048
    W, x = synth.small_case(40 + bits + group, N, K, 0.02, True)
    x = (x * np.exp2(np.arange(K) % 40 - 20)).astype(np.float32)
    err = _gemv_case(qg, oracle, W, x, bits, group, (0, 0, kernel))
    assert err <= TOL_FP32, err


def _awkward_x(kind, K, rng):
    x = rng.standard_normal(K).astype(np.float32)
    if kind == "zero runs":                 # whole steps of zeros between ordinary ones
        x[256:768] = 0.0
        x[K - 256:] = 0.0
    elif kind == "one nonzero per step":
        keep = x[::128].copy()
        x[:] = 0.0
        x[::128] = keep
    elif kind == "huge":                    # near the top of the fp32 range, both signs
        x *= np.float32(1e30)
    elif kind == "tiny":
        x *= np.float32(1e-25)
    elif kind == "spikes":                  # one element per step 2^20 above the rest
        x[5::256] *= np.float32(2.0 ** 20)
    elif kind == "negative peak":
        x = -np.abs(x)
        x[3::64] *= np.float32(1000.0)
    return x


@pytest.mark.parametrize("kind", ["zero runs", "one nonzero per step", "huge", "tiny", "spikes", "negative peak"])
@pytest.mark.parametrize("bits,group", [(4, 128), (4, 32), (3, 64), (2, 32), (2, 2048), (3, 1024), (4, 2048)])
@pytest.mark.parametrize("kernel", [0, 3])
def test_gemv_awkward_activations(qg, oracle, bits, group, kernel, kind):
    # inputs that stress how x enters the matrix instructions: the fixed point of a step follows
    # the largest |x| of that step (int8 form), the bf16 parts must carry signs and magnitudes
    _announce("gemv awkward x", bits, group, kernel, kind)
    N, K = 130, 2048
    W, _ = synth.small_case(90 + bits + group, N, K, 0.02, True)
    x = _awkward_x(kind, K, np.random.default_rng(17 + bits))
    err = _gemv_case(qg, oracle, W, x, bits, group, (0, 0, kernel))
    assert err <= TOL_FP32, err


@pytest.mark.parametrize("bits,group", [(4, 128), (3, 64), (2, 32), (4, 1024)])
@pytest.mark.parametrize("kernel", [0, 1, 3])
def test_gemv_non_finite_activations_reach_the_output(qg, bits, group, kernel):
    # a NaN or an infinity in x must not vanish in the conversion of x for the matrix instructions
    _announce("gemv non-finite x", bits, group, kernel)
    N, K = 130, 1024
    W, x = synth.small_case(3 + bits, N, K, 0.02, False)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    blob = qg.qg_pack(q, s, z, bits, group, qg.QG_LAYOUT_DEVICE)
    qg.qg_set_gemv_tuning(0, 0, kernel)
    try:
        for bad in (np.nan, np.inf, -np.inf):
            xb = x.copy()
            xb[517] = bad
            y = host(qg.qg_gemv(blob, N, K, bits, group, dev(xb)))
            assert not np.isfinite(y).any(), (bad, int(np.isfinite(y).sum()))
    finally:
        qg.qg_set_gemv_tuning(0, 0, 0)


@pytest.mark.parametrize("kernel", [0, 1, 3])
@pytest.mark.parametrize("bits,group", [(4, 128), (2, 32), (3, 1024)])
def test_gemv_nan_with_the_empty_slot_pattern(qg, bits, group, kernel):
    # The meeting slots of the K-split mark "empty" with the bit pattern 0xffffffff, itself a NaN.
    # An x element with exactly that pattern travels through the sums as a payload; the partial
    # result must still be taken for a value (and y written, as NaN), not for an empty slot.
    _announce("gemv NaN = slot marker", bits, group, kernel)
    N, K = 130, 4096
    W, x = synth.small_case(11 + bits, N, K, 0.02, False)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    blob = qg.qg_pack(q, s, z, bits, group, qg.QG_LAYOUT_DEVICE)
    xb = x.copy()
    xb.view(np.uint32)[1234] = 0xFFFFFFFF
    for tuning in ((2, 4096, kernel), (1, 8192, kernel), (0, 0, kernel)):      # K cut over 2 ... 16 workgroups, and the built-in shape
        qg.qg_set_gemv_tuning(*tuning)
        try:
            ws = qg.new_workspace(qg.qg_workspace_bytes(N, K, bits, group, 1))
            y = torch.full((N,), 7.0, dtype=torch.float32, device="cuda")
            qg.qg_gemv(blob, N, K, bits, group, dev(xb), y, ws)
            y_clean = qg.qg_gemv(blob, N, K, bits, group, dev(x), None, ws)    # the workspace is still usable
            torch.cuda.synchronize()
        finally:
            qg.qg_set_gemv_tuning(0, 0, 0)
        assert np.isnan(host(y)).all(), (tuning, int((host(y) == 7.0).sum()))
        assert np.all(host(ws) == 0xFF), "workspace not left in its prepared state"
        assert np.isfinite(host(y_clean)).all()


@pytest.mark.parametrize("H,K,bits,group", [(320, 1024, 4, 128), (4096, 4096, 4, 128), (192, 1536, 3, 64)])
def test_gemv_stacked_projections_equal_separate_ones(qg, oracle, H, K, bits, group):
    # q, k and v of a block as ONE 3H x K product (one launch, one x): quantization is per output
    # and group, so the stacked matrix packs the same codes, and its y is the three y one after
    # the other -- against the oracle, and against the three products as problems of a grouped launch
    _announce("gemv stacked q/k/v", H, K, bits, group)
    Ws = [synth.small_case(600 + i, H, K, 0.02, True)[0] for i in range(3)]
    _, x = synth.small_case(650, H, K, 0.02, False)
    W3 = np.concatenate(Ws, axis=0)
    q0, s0, z0 = oracle.quantize(W3, bits, group)
    y_ref = oracle.matvec(q0, s0, z0, group, x)
    norms = oracle.row_norms(q0, s0, z0, group)
    q, s, z = qg.qg_quantize(dev(W3), bits, group)
    assert np.array_equal(host(q), q0)
    y3 = host(qg.qg_gemv(qg.qg_pack(q, s, z, bits, group), 3 * H, K, bits, group, dev(x)))
    assert scaled_error(y3, y_ref, norms, x) <= TOL_FP32
    problems = []
    for i in range(3):
        qi, si, zi = qg.qg_quantize(dev(Ws[i]), bits, group)
        assert np.array_equal(host(qi), q0[i * H:(i + 1) * H])                 # same codes as in the stack
        problems.append(dict(packed=qg.qg_pack(qi, si, zi, bits, group), N=H, K=K, bits=bits, group=group,
                             x=dev(x), y=torch.empty(H, dtype=torch.float32, device="cuda")))
    ys = np.concatenate([host(y) for y in qg.qg_gemv_grouped(problems)])
    assert scaled_error(ys, y_ref, norms, x) <= TOL_FP32
    assert scaled_error(ys, y3.astype(np.float64), norms, x) <= 2e-6           # two fp32 summation orders apart at most


@pytest.mark.parametrize("tuning", [(1, 4096, 1), (2, 4096, 1), (4, 8192, 1), (8, 4096, 1), (16, 4096, 1), (4, 65536, 1),
                                    (1, 4096, 2), (3, 8192, 2), (8, 4096, 2), (16, 4096, 2), (4, 65536, 2),
                                    (1, 4096, 3), (3, 8192, 3), (8, 4096, 3), (4, 65536, 3),
                                    (1, 4096, 4), (3, 8192, 4), (8, 4096, 4), (4, 65536, 4)])
@pytest.mark.parametrize("N,K,bits,group", [(200, 4096, 4, 128), (130, 3072, 3, 64), (130, 4096, 2, 32),
                                            (70, 4096, 4, 1024), (70, 5632, 4, 5632), (70, 3840, 3, 1280),
                                            (70, 5632, 2, 2816), (130, 11008, 3, 11008)])
def test_gemv_k_split_shapes(qg, oracle, N, K, bits, group, tuning):
    # the same product under different wavefront / workgroup splits of K, including the
    # path where the last-arriving workgroup adds the partial vectors
    _announce("gemv split", N, K, bits, group, tuning)
    W, x = synth.small_case(N + K + bits, N, K, 0.02, False)
    err = _gemv_case(qg, oracle, W, x, bits, group, tuning)
    assert err <= TOL_FP32, err


@pytest.mark.parametrize("N,K,bits,group", [(70, 1 << 20, 4, 128),      # a very long K: 32 workgroups x 12 wavefronts per tile
                                            (70, 1 << 19, 2, 1 << 19),   # ... as one group per output
                                            (1 << 20, 128, 4, 128),      # a very long N: one step per tile
                                            (300000, 256, 3, 64)])
def test_gemv_extreme_shapes(qg, oracle, N, K, bits, group):
    _announce("gemv extreme", N, K, bits, group)
    W, x = synth.small_case(7 + bits, N, K, 0.02, False)
    err = _gemv_case(qg, oracle, W, x, bits, group)
    assert err <= TOL_FP32, err


@pytest.mark.parametrize("N,K,bits,group,tuning", [
    (70, 262144, 2, 16, (0, 0, 0)),      # a long K of tiny groups on the built-in choice
    (70, 294912, 2, 16, (0, 0, 0)),
    (70, 262144, 4, 16, (0, 0, 0)),
    (70, 294912, 4, 16, (0, 0, 1)),      # vector ALU: 64 groups per wavefront at most, 288 wavefronts per tile
    (70, 262144, 2, 16, (4, 0, 2)),      # 32 x 32 x 16 kernel: teams of 4 cannot cover K, the widest (8) can
    (70, 294912, 2, 16, (4, 0, 2)),      # ... nor can those: the vector-ALU kernel's teams of 16
    (130, 13824, 2, 16, (2, 0, 2)),      # a forced team size that cannot cover K without an empty workgroup
    (130, 13824, 2, 16, (1, 4096, 3)),
    (130, 13824, 3, 32, (1, 4096, 2))])
def test_gemv_team_size_fallback(qg, oracle, N, K, bits, group, tuning):
    # small groups limit the steps of a wavefront; a long K then needs more wavefronts per tile
    # than the preferred (or the forced) team size allows, and the launch widens the teams
    _announce("gemv team fallback", N, K, bits, group, tuning)
    W, x = synth.small_case(N + bits, N, K, 0.02, False)
    err = _gemv_case(qg, oracle, W, x, bits, group, tuning)
    assert err <= TOL_FP32, err


def test_calls_run_on_the_stream_they_are_given(qg, oracle):
    # every kernel of a call goes to the caller's stream: on a side stream (default priority) that is
    # held back by a long fill, the results are there after that stream alone has been waited for
    _announce("side stream")
    N, K, bits, group, M = 300, 4096, 4, 128, 24
    W, X = synth.small_case(1600, N, K, 0.02, True, m=M)
    q0, s0, z0 = oracle.quantize(W, bits, group)
    norms = oracle.row_norms(q0, s0, z0, group)
    y_ref = oracle.matvec(q0, s0, z0, group, X[0])
    Y_ref = oracle.matmul_small(q0, s0, z0, group, X)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    blob = qg.qg_pack(q, s, z, bits, group)
    Xd = dev(X)
    x0 = Xd[0].contiguous()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    ballast = torch.empty(64 << 20, dtype=torch.float32, device="cuda")
    with torch.cuda.stream(side):
        ws = qg.new_workspace(qg.qg_workspace_bytes(N, K, bits, group, 1))
        wsm = qg.new_workspace(qg.qg_workspace_bytes(N, K, bits, group, M))
        for _ in range(4):
            ballast.fill_(1.0)
        y = qg.qg_gemv(blob, N, K, bits, group, x0, None, ws)
        y2 = qg.qg_gemv_noalloc(blob, N, K, bits, group, x0, torch.empty(N, dtype=torch.float32, device="cuda"))
        narrow = qg.qg_to_narrow(blob, N, K, bits, group)
        yn = qg.qg_gemv_narrow(narrow, N, K, bits, group, x0)
        back = qg.qg_from_narrow(narrow, N, K, bits, group)
        Y = qg.qg_gemm_small(blob, N, K, bits, group, Xd, None, wsm)
        qg.qg_set_gemm_tuning(0, 13)
        try:
            Yc = qg.qg_gemm_small(blob, N, K, bits, group, Xd, None, wsm)
        finally:
            qg.qg_set_gemm_tuning(0, 0)
    side.synchronize()
    assert scaled_error(host(y), y_ref, norms, X[0]) <= TOL_FP32
    assert np.array_equal(host(y), host(y2))
    assert scaled_error(host(yn), y_ref, norms, X[0]) <= TOL_FP32
    assert np.array_equal(host(back), host(blob))
    assert scaled_error(host(Y), Y_ref, norms, X) <= gemm_model_bound(K)
    assert scaled_error(host(Yc), Y_ref, norms, X) <= gemm_model_bound(K)
    torch.cuda.synchronize()


def test_gemv_zero_input_and_unit_scale(qg, oracle):
    _announce("gemv x = 0, s = 1 z = 0")
    rng = np.random.default_rng(5)
    N, K, bits, group = 130, 512, 4, 64
    q = rng.integers(0, 16, (N, K), dtype=np.uint8)
    s = np.ones((N, K // group), np.float32)
    z = np.zeros((N, K // group), np.uint8)
    blob = qg.qg_pack(dev(q), dev(s), dev(z), bits, group, qg.QG_LAYOUT_DEVICE)
    y = qg.qg_gemv(blob, N, K, bits, group, torch.zeros(K, device="cuda"))
    assert not host(y).any()
    x = rng.integers(-8, 9, K).astype(np.float32)            # small integers: fp32 sums are exact
    y = host(qg.qg_gemv(blob, N, K, bits, group, dev(x)))
    assert np.array_equal(y.astype(np.int64), q.astype(np.int64) @ x.astype(np.int64))


def test_gemv_grouped_mixed_problems(qg, oracle):
    _announce("gemv grouped, mixed shapes and formats")
    specs = [(200, 1024, 4, 128), (130, 512, 4, 128), (64, 1536, 3, 64), (90, 480, 4, 24),
             (257, 1024, 2, 32), (512, 512, 4, 128), (100, 2048, 4, 2048),
             (70, 2304, 4, 768), (130, 5632, 4, 5632),       # long groups of different sizes share a launch
             (66, 1536, 3, 768), (77, 1024, 3, 64)]
    problems, refs = [], []
    for i, (N, K, bits, group) in enumerate(specs):
        W, x = synth.small_case(900 + i, N, K, 0.02, True)
        q0, s0, z0 = oracle.quantize(W, bits, group)
        refs.append((oracle.matvec(q0, s0, z0, group, x), oracle.row_norms(q0, s0, z0, group), x))
        q, s, z = qg.qg_quantize(dev(W), bits, group)
        problems.append(dict(packed=qg.qg_pack(q, s, z, bits, group), N=N, K=K, bits=bits, group=group,
                             x=dev(x), y=torch.empty(N, dtype=torch.float32, device="cuda")))
    ys = qg.qg_gemv_grouped(problems)
    torch.cuda.synchronize()
    for y, (y_ref, norms, x) in zip(ys, refs):
        assert scaled_error(host(y), y_ref, norms, x) <= TOL_FP32


@pytest.mark.parametrize("count", [12, 13, 14, 16])
def test_gemv_grouped_many_problems_of_one_format(qg, oracle, count):
    # one kernel launch with up to the maximum number of problems (the block table is searched
    # in two parts: twelve entries in registers, the rest from the argument buffer)
    _announce("gemv grouped, one format", count)
    problems, refs = [], []
    for i in range(count):
        N, K, bits, group = 64 + 37 * i, 512 + 128 * (i % 5), 4, 128
        W, x = synth.small_case(4000 + i, N, K, 0.02, False)
        q0, s0, z0 = oracle.quantize(W, bits, group)
        refs.append((oracle.matvec(q0, s0, z0, group, x), oracle.row_norms(q0, s0, z0, group), x))
        q, s, z = qg.qg_quantize(dev(W), bits, group)
        problems.append(dict(packed=qg.qg_pack(q, s, z, bits, group), N=N, K=K, bits=bits, group=group,
                             x=dev(x), y=torch.empty(N, dtype=torch.float32, device="cuda")))
    ys = qg.qg_gemv_grouped(problems)
    torch.cuda.synchronize()
    for y, (y_ref, norms, x) in zip(ys, refs):
        assert scaled_error(host(y), y_ref, norms, x) <= TOL_FP32


@pytest.mark.parametrize("I,K,bits,group,tuning", [(128, 512, 4, 128, (0, 0, 0)), (320, 1024, 4, 64, (0, 0, 0)),
                                                   (192, 4096, 4, 128, (2, 4096, 1)),      # K cut over workgroups
                                                   (256, 1536, 3, 64, (0, 0, 0)), (256, 1536, 3, 64, (0, 0, 1)),
                                                   (128, 2048, 2, 32, (0, 0, 0)), (64, 2048, 4, 2048, (0, 0, 0)),
                                                   (11008, 4096, 4, 128, (0, 0, 0))])     # LLaMA-7B gate/up
def test_gemv_swiglu_matches_oracle(qg, oracle, I, K, bits, group, tuning):
    _announce("gemv swiglu", I, K, bits, group, tuning)
    std = 0.02 if K < 4096 else 0.02
    W, x = synth.small_case(2000 + I + bits, 2 * I, K, std, True)
    q0, s0, z0 = oracle.quantize(W, bits, group)
    y_ref = oracle.matvec(q0, s0, z0, group, x)
    g, u = y_ref[:I], y_ref[I:]
    h_ref = oracle.swiglu(g, u)
    # what an error of TOL_FP32 * |row| * |x| in each product may do to h (|silu'| <= 1.1, |silu(g)| <= |g|)
    e = TOL_FP32 * oracle.row_norms(q0, s0, z0, group) * np.linalg.norm(x.astype(np.float64))
    tol = 1.1 * e[:I] * (np.abs(u) + e[I:]) + np.abs(g) * e[I:] + 1e-6 * np.abs(h_ref)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    blob = qg.qg_pack(q, s, z, bits, group)
    ws = qg.new_workspace(qg.qg_workspace_bytes(2 * I, K, bits, group, 1))
    qg.qg_set_gemv_tuning(*tuning)
    try:
        h = torch.full((I + 64,), 7.0, dtype=torch.float32, device="cuda")
        qg.qg_gemv_swiglu(blob, I, K, bits, group, dev(x), h[:I], ws)
        h2 = qg.qg_gemv_swiglu(blob, I, K, bits, group, dev(x), None, ws)          # workspace reuse
        y = host(qg.qg_gemv(blob, 2 * I, K, bits, group, dev(x)))                  # same launch shape
        torch.cuda.synchronize()
    finally:
        qg.qg_set_gemv_tuning(0, 0, 0)
    hh = host(h)
    assert np.all(hh[I:] == 7.0), "write past the end of h"
    assert np.array_equal(hh[:I], host(h2)), "not deterministic / workspace not left clean"
    assert np.all(host(ws) == 0xFF), "workspace not left in its prepared state"
    assert np.all(np.abs(hh[:I] - h_ref) <= tol), float(np.max(np.abs(hh[:I] - h_ref) / tol))
    # and it is the plain product (same split of K, so the same bits) followed by the elementwise step
    yg, yu = y[:I].astype(np.float64), y[I:].astype(np.float64)
    assert np.allclose(hh[:I], yg / (1.0 + np.exp(-yg)) * yu, rtol=2e-6, atol=1e-30)


def test_gemv_autotune_leaves_a_working_choice(qg, oracle):
    _announce("gemv autotune")
    specs = [(300, 2048, 4, 128), (200, 1024, 4, 128), (130, 4096, 4, 128)]
    problems, refs = [], []
    for i, (N, K, bits, group) in enumerate(specs):
        W, x = synth.small_case(1200 + i, N, K, 0.02, True)
        q0, s0, z0 = oracle.quantize(W, bits, group)
        refs.append((oracle.matvec(q0, s0, z0, group, x), oracle.row_norms(q0, s0, z0, group), x))
        q, s, z = qg.qg_quantize(dev(W), bits, group)
        problems.append(dict(packed=qg.qg_pack(q, s, z, bits, group), N=N, K=K, bits=bits, group=group,
                             x=dev(x), y=torch.empty(N, dtype=torch.float32, device="cuda")))
    launch = qg.GroupedGemv(problems)
    twin = qg.GroupedGemv([dict(p, packed=p["packed"].clone()) for p in problems], launch.workspace)
    try:
        wpb, bpw, kernel, us = qg.qg_gemv_autotune([launch, twin], repeats=6)
        assert wpb in (0, 2, 4, 8, 12, 16) and bpw in (0, 4096, 8192, 16384, 32768, 49152, 65536) and kernel in (1, 2, 3, 4) and us > 0
        # every candidate was either dropped by the resource budget or timed, and the installed
        # one is the fastest of those that were timed
        table, timed, dropped = qg.qg_gemv_autotune_report()
        assert timed + dropped == 168 and timed >= 1
        assert sum(1 for t in table if t > 0) == timed and sum(1 for t in table if t == -1.0) == dropped
        chosen = ((kernel - 1) * 6 + qg.AUTOTUNE_TEAMS.index(wpb)) * 7 + qg.AUTOTUNE_SIZES.index(bpw)
        assert table[chosen] > 0 and table[chosen] == min(t for t in table if t > 0)
        assert abs(table[chosen] - us) <= 1e-3 * us
        for p in problems:
            p["y"].fill_(7.0)
        launch.launch()
        torch.cuda.synchronize()
        for p, (y_ref, norms, x) in zip(problems, refs):
            assert scaled_error(host(p["y"]), y_ref, norms, x) <= TOL_FP32
        assert np.all(host(launch.workspace) == 0xFF)
    finally:
        qg.qg_set_gemv_tuning(0, 0, 0)
        qg.qg_clear_tuning()


def test_gemv_recorded_tuning_applies_to_its_shapes_only(qg, oracle):
    # a tuning recorded for one list of shapes is used by launches with exactly that list, by no
    # other launch, and not after qg_clear_tuning; the process-wide knobs still win
    _announce("gemv recorded tuning")
    N, K, bits, group = 300, 2048, 4, 128
    W, x = synth.small_case(1300, N, K, 0.02, True)
    q0, s0, z0 = oracle.quantize(W, bits, group)
    y_ref, norms = oracle.matvec(q0, s0, z0, group, x), oracle.row_norms(q0, s0, z0, group)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    blob = qg.qg_pack(q, s, z, bits, group)
    W2, x2 = synth.small_case(1301, 200, 1024, 0.02, True)
    q2, s2, z2 = qg.qg_quantize(dev(W2), bits, group)
    blob2 = qg.qg_pack(q2, s2, z2, bits, group)

    def run_a():
        y = qg.qg_gemv(blob, N, K, bits, group, dev(x))
        torch.cuda.synchronize()
        assert scaled_error(host(y), y_ref, norms, x) <= TOL_FP32
        return qg.qg_last_gemv_kernel()

    def run_b():
        qg.qg_gemv(blob2, 200, 1024, bits, group, dev(x2))
        torch.cuda.synchronize()
        return qg.qg_last_gemv_kernel()

    try:
        builtin_a, builtin_b = run_a(), run_b()
        assert builtin_a.startswith("gemv_mma4i") and builtin_b.startswith("gemv_mma4i")
        qg.qg_gemv_record_tuning([dict(N=N, K=K, bits=bits, group=group)], 8, 8192, 1)
        assert run_a().startswith("gemv_static")           # the vector-ALU kernel, as recorded
        assert run_b() == builtin_b                         # another shape: untouched
        both = [dict(packed=blob, N=N, K=K, bits=bits, group=group, x=dev(x), y=torch.empty(N, device="cuda")),
                dict(packed=blob2, N=200, K=1024, bits=bits, group=group, x=dev(x2), y=torch.empty(200, device="cuda"))]
        qg.qg_gemv_grouped(both)                            # another list of shapes: untouched
        torch.cuda.synchronize()
        assert qg.qg_last_gemv_kernel().startswith("gemv_mma4i")
        qg.qg_set_gemv_tuning(0, 0, 3)                      # the knobs win over the record
        assert run_a().startswith("gemv_mma4<")
        qg.qg_set_gemv_tuning(0, 0, 0)
        assert run_a().startswith("gemv_static")
        qg.qg_clear_tuning()
        assert run_a() == builtin_a
    finally:
        qg.qg_set_gemv_tuning(0, 0, 0)
        qg.qg_clear_tuning()


@pytest.mark.parametrize("N,K,bits,group,M", [(640, 2048, 4, 128, 24), (520, 1536, 3, 64, 70), (300, 1024, 2, 32, 16)])
def test_gemm_autotune_records_a_working_choice(qg, oracle, N, K, bits, group, M):
    _announce("gemm autotune", N, K, bits, group, M)
    W, X = synth.small_case(1400 + bits, N, K, 0.02, True, m=M)
    q0, s0, z0 = oracle.quantize(W, bits, group)
    Y_ref, norms = oracle.matmul_small(q0, s0, z0, group, X), oracle.row_norms(q0, s0, z0, group)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    blob = qg.qg_pack(q, s, z, bits, group)
    try:
        splits, shape, us = qg.qg_gemm_autotune([blob, blob.clone()], N, K, bits, group, dev(X), repeats=4)
        table, timed, dropped = qg.qg_gemm_autotune_report()
        assert 1 <= splits <= 8 and shape in qg.GEMM_AUTOTUNE_SHAPES and us > 0 and timed >= 1
        assert sum(1 for t in table if t > 0) == timed and sum(1 for t in table if t == -1.0) == dropped
        chosen = qg.GEMM_AUTOTUNE_SHAPES.index(shape) * 8 + splits - 1
        assert table[chosen] > 0 and table[chosen] == min(t for t in table if t > 0)
        # the recorded choice is what the next call runs, and it is a correct one
        Y = qg.qg_gemm_small(blob, N, K, bits, group, dev(X))
        torch.cuda.synchronize()
        err = scaled_error(host(Y), Y_ref, norms, X)
        assert err <= TOL_BF16 and err <= gemm_model_bound(K), err
        qg.qg_set_gemm_tuning(splits, shape)                 # the same choice through the knobs: same bits
        Y2 = qg.qg_gemm_small(blob, N, K, bits, group, dev(X))
        torch.cuda.synchronize()
        assert np.array_equal(host(Y), host(Y2))
    finally:
        qg.qg_set_gemm_tuning(0, 0)
        qg.qg_clear_tuning()


# ------------------------------------------------------------------ full benchmark sizes

FULL = [("C2", 0), ("C2", 4), ("C2", 6), ("C3", 0), ("C3", 4), ("C3", 6), ("C4", 0), ("C4", 4), ("C4", 6)]


@pytest.mark.parametrize("name,index", FULL)
def test_full_size_matrix(qg, oracle, name, index):
    # every distinct shape of the three layer sets, at full size, all outputs compared
    cfg = synth.CONFIGS[name]
    N, K = cfg.shapes[index]
    _announce("full size", name, index, N, K, cfg.bits, cfg.group)
    W, (x,) = synth.matrix(cfg, index)
    q0, s0, z0 = oracle.quantize(W, cfg.bits, cfg.group)
    Wd = dev(W)
    del W
    q, s, z = qg.qg_quantize(Wd, cfg.bits, cfg.group)
    del Wd
    assert np.array_equal(host(q), q0)
    assert np.array_equal(host(s).view(np.uint32), s0.view(np.uint32))
    assert np.array_equal(host(z), z0)
    blob = qg.qg_pack(q, s, z, cfg.bits, cfg.group)
    q2, s2, z2 = qg.qg_unpack(blob, N, K, cfg.bits, cfg.group)
    assert torch.equal(q2, q) and torch.equal(z2, z) and torch.equal(s2.view(torch.int32), s.view(torch.int32))
    y = host(qg.qg_gemv(blob, N, K, cfg.bits, cfg.group, dev(x)))
    y_ref = oracle.matvec(q0, s0, z0, cfg.group, x)
    err = scaled_error(y, y_ref, oracle.row_norms(q0, s0, z0, cfg.group), x)
    print(f"[full] {name}[{index}] scaled error {err:.3e}", flush=True)
    assert err <= TOL_FP32, err


def _random_format(rng):
    bits = int(rng.choice([2, 3, 4]))
    cell = {4: 8, 2: 16, 3: 32}[bits]
    mult = int(rng.choice([1, 1, 2, 4, 4, 8, 16]))
    group = cell * mult
    if bits == 3 and mult == 16:
        group = 256
    return bits, group


@pytest.mark.parametrize("seed", range(6))
def test_gemv_random_shapes_and_launch_shapes(qg, oracle, seed):
    # seeded sweep over the launch-shape logic: ragged N, K from one group to many steps, every
    # format, team sizes / bytes per wavefront / kernel picked at random
    rng = np.random.default_rng(7000 + seed)
    for case in range(8):
        bits, group = _random_format(rng)
        ngroups = int(rng.integers(1, 1 + max(1, 6000 // group)))
        if rng.random() < 0.2:
            group, ngroups = group * ngroups, 1                     # one group per output
            if group > 8192:
                group = 8192 // ({4: 8, 2: 16, 3: 32}[bits]) * ({4: 8, 2: 16, 3: 32}[bits])
        K = group * ngroups
        N = int(rng.integers(1, 400))
        tuning = (int(rng.choice([0, 1, 2, 4, 7, 8, 12, 16])), int(rng.choice([0, 4096, 8192, 16384, 65536])),
                  int(rng.choice([0, 1, 2, 3, 4])))
        _announce("gemv random", seed, case, N, K, bits, group, tuning)
        W, x = synth.small_case(seed * 100 + case, N, K, 0.02, bool(rng.integers(0, 2)))
        err = _gemv_case(qg, oracle, W, x, bits, group, tuning)
        assert err <= TOL_FP32, (N, K, bits, group, tuning, err)


# ------------------------------------------------------------------ small-M GEMM (bf16 MFMA path)

TOL_BF16 = 1e-2


def gemm_model_bound(K):
    """What the rounding of both operands to bf16 may cost, as a multiple of |What[n,:]| |X[m,:]|.
    Round-to-nearest to 8 significant bits errs by at most 2^-8 relative, 0.42 * 2^-8 rms for a
    log-uniform significand; two rounded operands per product: 2.3e-3 rms per term; the terms'
    errors are independent, so the sum errs by 2.3e-3 * sqrt(sum (x w)^2) = 2.3e-3 / sqrt(K) of
    |w| |x| for activations that are independent of the weights; the largest of up to a million
    outputs lies near 5 sigma: 1.2e-2 / sqrt(K) = 6.1 * 2^-9 / sqrt(K).  The bound is that with a
    margin of 2.6: c = 16.  (A kernel that keeps the codes exact and rounds only X stays a factor
    sqrt(2) further inside.)  fp32 accumulation adds sqrt(K) * 2^-24, far below."""
    return 16.0 * 2.0 ** -9 / np.sqrt(K)


def _gemm_case(qg, oracle, W, X, bits, group):
    N, K = W.shape
    M = X.shape[0]
    q0, s0, z0 = oracle.quantize(W, bits, group)
    Y_ref = oracle.matmul_small(q0, s0, z0, group, X)
    norms = oracle.row_norms(q0, s0, z0, group)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    blob = qg.qg_pack(q, s, z, bits, group, qg.QG_LAYOUT_DEVICE)
    ws = qg.new_workspace(qg.qg_workspace_bytes(N, K, bits, group, M))
    Y = torch.full((M * N + 64,), 7.0, dtype=torch.float32, device="cuda")      # canary behind Y
    qg.qg_gemm_small(blob, N, K, bits, group, dev(X), Y[:M * N].view(M, N), ws)
    Y2 = qg.qg_gemm_small(blob, N, K, bits, group, dev(X), None, ws)            # workspace reuse
    torch.cuda.synchronize()
    Yh = host(Y)
    assert np.all(Yh[M * N:] == 7.0), "write past the end of Y"
    assert np.array_equal(Yh[:M * N].reshape(M, N), host(Y2)), "not deterministic"
    err = scaled_error(Yh[:M * N].reshape(M, N), Y_ref, norms, X)
    # next to the caller's 1e-2: the level the rounding model allows at this K (Gaussian X)
    assert err <= gemm_model_bound(K), (err, gemm_model_bound(K))
    return err


GEMM_CASES = [  # N, K, bits, group, M
    (256, 512, 4, 128, 16),
    (200, 1024, 4, 128, 5),      # ragged N and M
    (130, 768, 4, 64, 33),
    (70, 512, 4, 32, 100),
    (300, 1024, 4, 256, 64),
    (128, 2048, 4, 2048, 128),   # one group per output
    (64, 128, 4, 128, 1),
    (200, 640, 4, 128, 16),      # 5 steps: ragged last iteration of four k-slices
    (330, 1152, 4, 384, 20),     # group of three steps against four k-slices
    (190, 1408, 4, 64, 40),      # 11 steps against two k-slices, odd number of tiles
    (190, 1408, 4, 128, 128),
    (200, 1024, 4, 128, 65),     # second block of rows holds a single row
    (1100, 256, 4, 128, 72),     # enough tiles for the four-tile workgroup shape
    (130, 512, 3, 64, 7),        # other widths: fp32 row-by-row path
    (96, 512, 2, 32, 4),
    (90, 480, 4, 24, 3),
    (130, 1280, 3, 64, 37),      # more rows than one grouped launch of the row-by-row path holds
    (200, 512, 2, 16, 16),
]


@pytest.mark.parametrize("shape", [0, 13])       # the built-in choice / the raw-code kernel wherever it applies
@pytest.mark.parametrize("N,K,bits,group,M", GEMM_CASES)
def test_gemm_small_matches_oracle(qg, oracle, N, K, bits, group, M, shape):
    _announce("gemm_small", N, K, bits, group, M, shape)
    W, X = synth.small_case(N + K + M, N, K, 0.02, True, m=max(M, 2))
    X = X[:M]
    qg.qg_set_gemm_tuning(0, shape)
    try:
        err = _gemm_case(qg, oracle, W, X, bits, group)
    finally:
        qg.qg_set_gemm_tuning(0, 0)
    assert err <= TOL_BF16, err


CODES_CASES = [  # N, K, bits, group, M   -- the raw-code kernel: every group pattern of every width
    (200, 1024, 2, 32, 16), (130, 1024, 2, 64, 33), (96, 768, 2, 128, 7), (70, 1024, 2, 256, 100),
    (200, 1024, 2, 512, 64), (130, 1536, 2, 1536, 128),             # groups of whole steps, one group per output
    (200, 1024, 3, 64, 16), (130, 1536, 3, 128, 70), (96, 768, 3, 256, 5), (70, 2048, 3, 512, 128),
    (130, 1280, 3, 1280, 40),
    (200, 1024, 4, 16, 16), (130, 768, 4, 32, 50), (64, 512, 4, 64, 128), (300, 1024, 4, 128, 33),
    (128, 2048, 4, 2048, 128), (330, 1152, 4, 384, 20),
    (190, 1312, 3, 32 * 41, 9),      # K not a whole number of steps (padded), one group per output: row-by-row path
    (190, 1312, 2, 32, 9),           # K = 5 steps + 32: the last step is mostly padding
    (100, 416, 4, 32, 60),           # 3 steps + 32
    (1100, 512, 2, 32, 128), (1100, 512, 3, 64, 128),                # many tiles, two blocks of rows
]


@pytest.mark.parametrize("splits", [0, 1, 3])
@pytest.mark.parametrize("N,K,bits,group,M", CODES_CASES)
def test_gemm_small_raw_code_kernel(qg, oracle, N, K, bits, group, M, splits):
    _announce("gemm raw codes", N, K, bits, group, M, splits)
    W, X = synth.small_case(4000 + N + K + M, N, K, 0.02, True, m=max(M, 2))
    X = X[:M]
    qg.qg_set_gemm_tuning(splits, 13)
    try:
        err = _gemm_case(qg, oracle, W, X, bits, group)
    finally:
        qg.qg_set_gemm_tuning(0, 0)
    assert err <= TOL_BF16, err


@pytest.mark.parametrize("tuning", [(0, 0, 0), (1, 4096, 0), (3, 8192, 0), (8, 65536, 0)])
@pytest.mark.parametrize("N,K,group,M", [(200, 1024, 128, 16), (130, 512, 16, 7), (70, 1408, 32, 1), (300, 2304, 64, 13),
                                         (64, 11008, 128, 16), (1000, 128, 128, 9)])
def test_gemm_small_up_to_16_rows(qg, oracle, N, K, group, M, tuning):
    # the barrier-free kernel for a few rows: every group size it takes, ragged N and M, one
    # step, long K over a team of wavefronts, different team sizes
    _announce("gemm rows16", N, K, group, M, tuning)
    W, X = synth.small_case(3000 + N + M, N, K, 0.02, True, m=max(M, 2))
    X = X[:M]
    qg.qg_set_gemv_tuning(*tuning)
    qg.qg_set_gemm_tuning(0, -1)                 # this kernel whatever the number of tiles
    try:
        err = _gemm_case(qg, oracle, W, X, 4, group)
    finally:
        qg.qg_set_gemv_tuning(0, 0, 0)
        qg.qg_set_gemm_tuning(0, 0)
    assert err <= TOL_BF16, err


@pytest.mark.parametrize("bits,group,cell", [(4, 128, 8), (4, 32, 8), (3, 64, 32), (2, 32, 16)])
@pytest.mark.parametrize("M", [1, 16, 40, 128])
def test_gemm_small_single_cell_difference(qg, oracle, bits, group, cell, M):
    # Two outputs whose codes agree everywhere except in ONE cell (the smallest granule the kernels
    # decode): the difference of their results is that cell's contribution alone, far below the
    # 1e-2 bound on either result.  A cell that is dropped, doubled or paired with the wrong x
    # shows up here at full size.  Cells at the start, inside and at the end of K, in the first
    # and in a later tile.
    _announce("gemm single cell", bits, group, M)
    N, K = 200, 2048
    rng = np.random.default_rng(77 + bits + M)
    base = rng.integers(0, 1 << bits, K, dtype=np.uint8)
    q = np.tile(base, (N, 1))
    s = np.full((N, K // group), 0.03125, np.float32)
    z = np.full((N, K // group), (1 << bits) // 2, np.uint8)
    spots = [(1, 0), (5, K // cell - 1), (70, 3), (131, K // cell // 2 + 1), (199, K // cell - 2)]   # (output, cell)
    for n, c in spots:
        q[n, c * cell:(c + 1) * cell] = ((1 << bits) - 1) - q[n, c * cell:(c + 1) * cell]
    X = rng.standard_normal((max(M, 2), K)).astype(np.float32)[:M]
    blob = qg.qg_pack(dev(q), dev(s), dev(z), bits, group)
    Y = host(qg.qg_gemm_small(blob, N, K, bits, group, dev(X))).astype(np.float64)
    Y_ref = oracle.matmul_small(q, s, z, group, X)
    assert scaled_error(Y, Y_ref, oracle.row_norms(q, s, z, group), X) <= gemm_model_bound(K)
    xn = np.linalg.norm(X.astype(np.float64), axis=1)
    wn = float(oracle.row_norms(q, s, z, group)[0])
    for n, c in spots:
        d = Y[:, n] - Y[:, 0]                       # output 0 carries the unchanged codes
        d_ref = Y_ref[:, n] - Y_ref[:, 0]
        dq = q[n, c * cell:(c + 1) * cell].astype(np.float64) - base[c * cell:(c + 1) * cell]
        size = 0.03125 * np.linalg.norm(dq) * np.linalg.norm(X[:, c * cell:(c + 1) * cell].astype(np.float64), axis=1)
        # the cell's own terms rounded to bf16 (2^-8 each, two operands) plus fp32 accumulation of two long sums
        slack = 2.0 ** -7 * size + 8 * np.sqrt(K) * 2.0 ** -24 * wn * xn
        assert np.all(np.abs(d - d_ref) <= slack), (n, c, float(np.max(np.abs(d - d_ref) / slack)))
        assert np.all(np.abs(d_ref) > 0)


def test_gemm_small_longest_k_of_the_matrix_core_path(qg, oracle):
    _announce("gemm_small K = 2^20")
    N, K, bits, group, M = 70, 1 << 20, 4, 128, 9
    W, X = synth.small_case(31, N, K, 0.02, False, m=M)
    err = _gemm_case(qg, oracle, W, X, bits, group)
    assert err <= TOL_BF16, err


def test_gemm_small_rows_agree_with_gemv(qg, oracle):
    _announce("gemm_small rows vs gemv")
    N, K, bits, group, M = 256, 1024, 4, 128, 16
    W, X = synth.small_case(77, N, K, 0.02, True, m=M)
    q, s, z = qg.qg_quantize(dev(W), bits, group)
    blob = qg.qg_pack(q, s, z, bits, group)
    Y = host(qg.qg_gemm_small(blob, N, K, bits, group, dev(X)))
    q0, s0, z0 = oracle.quantize(W, bits, group)
    norms = oracle.row_norms(q0, s0, z0, group)
    for m in (0, 7, 15):
        y = host(qg.qg_gemv(blob, N, K, bits, group, dev(X[m])))
        assert scaled_error(Y[m], y.astype(np.float64), norms, X[m]) <= TOL_BF16


@pytest.mark.parametrize("splits", [1, 2, 3, 8])
@pytest.mark.parametrize("M", [24, 48, 96])
def test_gemm_small_every_split_count(qg, oracle, splits, M):
    _announce("gemm_small splits", splits, M)
    N, K, bits, group = 200, 2304, 4, 128          # 18 steps
    W, X = synth.small_case(500 + M, N, K, 0.02, True, m=M)
    qg.qg_set_gemm_tuning(splits, 0)
    try:
        err = _gemm_case(qg, oracle, W, X, bits, group)
    finally:
        qg.qg_set_gemm_tuning(0, 0)
    assert err <= TOL_BF16, err


@pytest.mark.parametrize("shape", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12])
@pytest.mark.parametrize("N,K,group", [(610, 1408, 64), (130, 1152, 384), (200, 128, 32), (70, 2560, 128)])
def test_gemm_small_every_workgroup_shape(qg, oracle, shape, N, K, group):
    # shapes 1-3 hold up to 32 rows, 4-7 blocks of 64 rows, 8-9 up to 64 rows in one wavefront,
    # 10-11 up to 128; ragged tiles and rows, odd and even numbers of steps, a single step
    M = 23 if shape <= 3 else 77 if shape <= 7 else 50 if shape in (8, 9, 12) else 101
    _announce("gemm_small shape", shape, N, K, group, M)
    W, X = synth.small_case(900 + shape, N, K, 0.02, True, m=M)
    for splits in (0, 2):
        qg.qg_set_gemm_tuning(splits, shape)
        try:
            err = _gemm_case(qg, oracle, W, X, 4, group)
        finally:
            qg.qg_set_gemm_tuning(0, 0)
        assert err <= TOL_BF16, (splits, err)


@pytest.mark.parametrize("seed", range(4))
def test_gemm_small_random_shapes(qg, oracle, seed):
    # seeded sweep: ragged N, M and step counts, the group sizes of the matrix-core path, split
    # counts and workgroup shapes picked at random (a shape that does not fit M is ignored)
    rng = np.random.default_rng(8000 + seed)
    for case in range(6):
        group = int(rng.choice([32, 64, 128, 128, 256, 384]))
        steps = int(rng.integers(1, 24))
        K = 128 * steps
        if K % group:
            K = group * max(1, K // group)
            if K % 128:
                K *= 128 // np.gcd(K, 128)
        N = int(rng.integers(1, 700))
        M = int(rng.integers(1, 129))
        splits, shape = int(rng.integers(0, 9)), int(rng.integers(0, 13))
        _announce("gemm random", seed, case, N, K, group, M, splits, shape)
        W, X = synth.small_case(seed * 100 + case + 50, N, K, 0.02, True, m=max(M, 2))
        qg.qg_set_gemm_tuning(splits, shape)
        try:
            err = _gemm_case(qg, oracle, W, X[:M], 4, group)
        finally:
            qg.qg_set_gemm_tuning(0, 0)
        assert err <= TOL_BF16, (N, K, group, M, splits, shape, err)


@pytest.mark.parametrize("seed", range(4))
def test_gemm_small_raw_code_random_shapes(qg, oracle, seed):
    # seeded sweep of the raw-code kernel over the three widths: groups of 2 ... 16 cells inside a
    # step and of 1 ... 3 whole steps, K that ends inside a step, ragged N and M, every count of
    # K ranges
    rng = np.random.default_rng(8100 + seed)
    for case in range(7):
        bits = int(rng.choice([2, 3, 4]))
        cell, step = {2: (16, 256), 3: (32, 256), 4: (8, 128)}[bits]
        cells_per_step = step // cell
        inside = [c * cell for c in (2, 4, 8, 16) if cells_per_step % c == 0]
        group = int(rng.choice(inside + [step, 2 * step, 3 * step]))
        K = group * int(rng.integers(1, max(2, 3072 // group)))
        if K % 16:
            K *= 16 // np.gcd(K, 16)
        N = int(rng.integers(1, 600))
        M = int(rng.integers(2, 129))
        splits = int(rng.integers(0, 9))
        _announce("gemm raw codes random", seed, case, N, K, bits, group, M, splits)
        W, X = synth.small_case(seed * 100 + case + 70, N, K, 0.02, True, m=M)
        qg.qg_set_gemm_tuning(splits, 13)
        try:
            err = _gemm_case(qg, oracle, W, X, bits, group)
        finally:
            qg.qg_set_gemm_tuning(0, 0)
        assert err <= TOL_BF16, (N, K, bits, group, M, splits, err)


@pytest.mark.parametrize("shape", [0, 13])
@pytest.mark.parametrize("index", [0, 1, 2])
@pytest.mark.parametrize("mi", [0, 1, 2])
def test_gemm_small_full_size(qg, oracle, index, mi, shape):
    # configuration 5: LLaMA-7B shapes, 4-bit group 128, M = 16, 64, 128; all outputs compared;
    # on the built-in choice of kernel and on the raw-code kernel
    cfg = synth.CONFIGS["C5"]
    N, K = cfg.shapes[index]
    M = cfg.batch[mi]
    _announce("gemm full size", N, K, M, shape)
    W, acts = synth.matrix(cfg, index)
    X = acts[mi]
    qg.qg_set_gemm_tuning(0, shape)
    try:
        err = _gemm_case(qg, oracle, W, X, cfg.bits, cfg.group)
    finally:
        qg.qg_set_gemm_tuning(0, 0)
    print(f"[full] C5[{index}] M={M} shape {shape} scaled error {err:.3e}", flush=True)
    assert err <= TOL_BF16, err


@pytest.mark.parametrize("name,index,M", [("C3", 0, 16), ("C3", 6, 128), ("C4", 0, 64), ("C4", 4, 16)])
def test_gemm_small_full_size_other_widths(qg, oracle, name, index, M):
    # 3-bit group 64 and 2-bit group 32 at the sizes of the 13B- and 65B-shaped layer sets
    cfg = synth.CONFIGS[name]
    N, K = cfg.shapes[index]
    _announce("gemm full size", name, N, K, M)
    W, _ = synth.matrix(cfg, index)
    X = np.random.Generator(np.random.Philox(77 + M)).standard_normal((M, K), dtype=np.float32)
    err = _gemm_case(qg, oracle, W, X, cfg.bits, cfg.group)
    print(f"[full] {name}[{index}] M={M} scaled error {err:.3e}", flush=True)
    assert err <= TOL_BF16, err


# ------------------------------------------------------------------ the benchmark's own launch

@pytest.mark.parametrize("name", ["C2", "C3", "C4"])
def test_layer_set_grouped_launch_full_size(qg, oracle, name):
    # the whole layer set in ONE grouped launch, as bench.py times it; every output of every
    # matrix is compared with the oracle
    cfg = synth.CONFIGS[name]
    _announce("grouped layer set", name)
    problems, refs = [], []
    for i, (N, K) in enumerate(cfg.shapes):
        W, (x,) = synth.matrix(cfg, i)
        q0, s0, z0 = oracle.quantize(W, cfg.bits, cfg.group)
        refs.append((oracle.matvec(q0, s0, z0, cfg.group, x), oracle.row_norms(q0, s0, z0, cfg.group), x))
        q, s, z = qg.qg_quantize(dev(W), cfg.bits, cfg.group)
        del W
        assert np.array_equal(host(q), q0) and np.array_equal(host(z), z0)
        assert np.array_equal(host(s).view(np.uint32), s0.view(np.uint32))
        problems.append(dict(packed=qg.qg_pack(q, s, z, cfg.bits, cfg.group), N=N, K=K, bits=cfg.bits,
                             group=cfg.group, x=dev(x), y=torch.empty(N, dtype=torch.float32, device="cuda")))
        del q, s, z, q0, s0, z0
    launch = qg.GroupedGemv(problems)
    launch.launch()
    first = [host(p["y"]).copy() for p in problems]
    launch.launch()                                              # same workspace again
    torch.cuda.synchronize()
    worst = 0.0
    for p, y1, (y_ref, norms, x) in zip(problems, first, refs):
        assert np.array_equal(host(p["y"]), y1), "not deterministic"
        worst = max(worst, scaled_error(y1, y_ref, norms, x))
    print(f"[full] {name} grouped launch, worst scaled error {worst:.3e}", flush=True)
    assert worst <= TOL_FP32, worst
