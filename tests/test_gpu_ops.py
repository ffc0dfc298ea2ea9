"""Parity of each HIP kernel, called through the C ABI, against the CPU oracle."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
import paper_2306_13835_amd as P
from paper_2306_13835_amd import binding as B
from oracle import opt_shard as O
from gpu_util import dev

pytestmark = pytest.mark.gpu


class Hooks:
    """An explicit list of switch values (see ctn_debug_gemm_tile) for ctn_test_op_gemm: the product runs under
    exactly these, applied in order to the library's defaults; nothing outlives the call."""

    def __init__(self):
        self.values = []

    def set(self, cfg):
        self.values.append(int(cfg))

    def gemm(self, A, W, bias, out, M, N, K, epi, stream, ws=None):
        B.test_op_gemm(A, W, bias, out, M, N, K, epi, ws, self.values, stream)


@pytest.fixture(scope="module")
def stream():
    torch.cuda.set_device(0)
    return torch.cuda.Stream()


def f16(rng, shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float16)


@pytest.mark.parametrize("nbytes", [16, 2560, 32 * 1024, 32 * 1024 + 16, 5 * 1024 * 1024 + 48])
@pytest.mark.parametrize("blocks", [1, 7, 64])
def test_copy_kernel_both_directions(stream, nbytes, blocks):
    pool = P.HostPool(2 * nbytes + 1024)
    try:
        src = pool.take((nbytes,), np.uint8)
        back = pool.take((nbytes,), np.uint8)
        rng = np.random.default_rng(nbytes)
        src[:] = rng.integers(0, 256, nbytes, dtype=np.uint8)
        back[:] = 0
        d = torch.full((nbytes + 512,), 0x7E, dtype=torch.uint8, device="cuda")
        B.op_copy(d.data_ptr() + 256, src, nbytes, blocks, stream)       # host -> device
        stream.synchronize()
        got = d.cpu().numpy()
        assert np.array_equal(got[256:256 + nbytes], src)
        assert (got[:256] == 0x7E).all() and (got[256 + nbytes:] == 0x7E).all()   # nothing outside the range
        B.op_copy(back, d.data_ptr() + 256, nbytes, blocks, stream)      # device -> host
        stream.synchronize()
        assert np.array_equal(back, src)
    finally:
        pool.close()


def test_copy_rejects_misaligned(stream):
    d = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(P.CtnError):
        B.op_copy(d.data_ptr(), d.data_ptr() + 512, 24, 1, stream)
    with pytest.raises(P.CtnError):
        B.op_copy(d.data_ptr() + 8, d.data_ptr() + 512, 32, 1, stream)


@pytest.mark.parametrize("hidden,rank,tp", [(768, 0, 1), (4096, 1, 2), (5120, 3, 4), (128, 0, 2)])
def test_embed(stream, hidden, rank, tp):
    rng = np.random.default_rng(hidden + rank)
    vocab, seq, batch = 512, 7, 3
    vl = vocab // tp
    tok, pos = f16(rng, (vl, hidden)), f16(rng, (seq + 2, hidden))
    ids = rng.integers(0, vocab, (batch, seq)).astype(np.int32)
    ids[0, 0], ids[0, 1] = rank * vl, (rank + 1) * vl - 1          # slice edges
    want = O.embed(ids, tok, pos, rank, np.float32).reshape(batch * seq, hidden)
    x = torch.empty(batch * seq, hidden, dtype=torch.float32, device="cuda")
    B.op_embed(dev(ids), dev(tok), dev(pos), x, batch * seq, seq, hidden, vl, rank, stream)
    stream.synchronize()
    assert np.array_equal(x.cpu().numpy(), want)                    # one fp32 add: exact


@pytest.mark.parametrize("rows,hidden", [(1, 768), (8, 768), (5, 2048), (133, 4096), (64, 5120), (3, 128), (9, 8192),
                                         (300, 4096), (257, 5120), (256, 2048), (700, 768),    # (more than 256 rows: the four-wavefront kernel)
                                         (7, 9216), (260, 9216), (64, 12288), (300, 12288), (5, 16384), (258, 16384),
                                         (3, 10240), (270, 14336)])    # (rows wider than 8192: three or four vectors per thread)
def test_layernorm(stream, rows, hidden):
    rng = np.random.default_rng(rows * hidden)
    x = (rng.standard_normal((rows, hidden)) * 3 + 0.5).astype(np.float32)
    g, b = (1 + 0.1 * rng.standard_normal(hidden)).astype(np.float16), f16(rng, hidden, 0.1)
    want = O.layer_norm(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64))
    out = torch.empty(rows, hidden, dtype=torch.float16, device="cuda")
    B.op_layernorm(dev(x), dev(g), dev(b), out, rows, hidden, stream)
    stream.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    # fp32 arithmetic then one rounding to fp16: within one fp16 ulp of the exact value
    assert np.all(np.abs(got - want) <= 2.0 ** -10 * np.maximum(np.abs(want), 2.0 ** -14) + 1e-6)


@pytest.mark.parametrize("rows,hidden", [(4, 4096), (300, 5120)])
def test_layernorm_rows_with_outliers(stream, rows, hidden):
    """Rows shaped like a trained decoder's residual stream: a few channels hundreds of times larger than the
    rest and a large common offset.  The two-pass variance (mean first, then centred squares) must hold the
    same bar as on well-behaved rows; a one-pass E[x^2] - E[x]^2 in fp32 would not."""
    rng = np.random.default_rng(rows + hidden)
    x = rng.standard_normal((rows, hidden)).astype(np.float32) + 40.0
    cols = rng.choice(hidden, 6, replace=False)
    x[:, cols] += (rng.standard_normal((rows, 6)) * 800.0).astype(np.float32)
    g, b = (1 + 0.1 * rng.standard_normal(hidden)).astype(np.float16), f16(rng, hidden, 0.1)
    want = O.layer_norm(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64))
    out = torch.empty(rows, hidden, dtype=torch.float16, device="cuda")
    B.op_layernorm(dev(x), dev(g), dev(b), out, rows, hidden, stream)
    stream.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    # the subtraction x - mean loses up to ulp_fp32(|x|) / std of relative accuracy on the small channels
    slack = 2.0 ** -23 * np.abs(x).max() / x.std(axis=1).min() * 4
    assert np.all(np.abs(got - want) <= 2.0 ** -10 * np.maximum(np.abs(want), 2.0 ** -14) + 1e-6 + slack)


def test_attention_peaked_scores(stream):
    """Scores tens of units apart (one key dominates every row, as in a trained model's sharp heads): the
    running maximum keeps every exponent at or below zero and the result stays within the bar."""
    rng = np.random.default_rng(77)
    batch, seq, heads, d = 2, 200, 4, 128
    hl = heads * d
    qkv = f16(rng, (batch * seq, 3 * hl), 1.0)
    qkv[:, :hl] *= np.float16(6.0)                       # q: scores ~ N(0, 6^2 * 128) / sqrt(128) -> spread of about 6, tails past 25
    q, k, v = (qkv[:, i * hl:(i + 1) * hl].astype(np.float64).reshape(batch, seq, hl) for i in range(3))
    want = O.attention(q, k, v, heads).reshape(batch * seq, hl)
    out = torch.full((batch * seq, hl), float("nan"), dtype=torch.float16, device="cuda")
    B.op_attention(dev(qkv), out, batch, seq, heads, d, stream)
    stream.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= 4e-3 * max(1.0, np.abs(want).max())
    assert np.abs(got - want).mean() <= 4e-4 * np.abs(want).mean() + 1e-5


GEMM_SHAPES = [(8, 520, 4104), (16, 77, 5120), (3, 4096, 8192), (1, 33, 4096), (8, 2304, 768), (1, 128, 64), (33, 200, 72), (16, 50, 40), (17, 4096, 2048), (48, 33, 8192), (49, 640, 264), (64, 6144, 4096), (130, 257, 136),
               (1024, 4096, 2048), (300, 50272 // 4, 512), (2048, 1280, 5120)]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("epi", [P.EPI_BIAS_F16, P.EPI_BIAS_RELU_F16, P.EPI_BIAS_RESID_F32, P.EPI_F32])
def test_gemm(stream, M, N, K, epi):
    rng = np.random.default_rng(M * 31 + N * 7 + K + epi)
    A, W, bias = f16(rng, (M, K)), f16(rng, (N, K), 0.05), f16(rng, N, 0.5)
    res = rng.standard_normal((M, N)).astype(np.float32)
    acc = A.astype(np.float64) @ W.astype(np.float64).T     # the definition, in fp64 on the CPU
    if epi == P.EPI_BIAS_F16:
        want, out = acc + bias.astype(np.float64), torch.empty(M, N, dtype=torch.float16, device="cuda")
    elif epi == P.EPI_BIAS_RELU_F16:
        want, out = np.maximum(acc + bias.astype(np.float64), 0), torch.empty(M, N, dtype=torch.float16, device="cuda")
    elif epi == P.EPI_BIAS_RESID_F32:
        want, out = res + acc + bias.astype(np.float64), dev(res)
    else:
        want, out = acc, torch.empty(M, N, dtype=torch.float32, device="cuda")
    guard = torch.full((4096,), 7.0, dtype=torch.float32, device="cuda")   # detect stray writes after `out`
    B.op_gemm(dev(A), dev(W), dev(bias), out, M, N, K, epi, stream)
    stream.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    scale = np.sqrt(K) * 0.05
    if out.dtype == torch.float16:
        assert np.all(np.abs(got - want) <= 2.0 ** -10 * np.abs(want) + 1e-4 * scale + 1e-7)
    else:
        assert np.abs(got - want).max() <= 2e-5 * scale * max(1.0, np.log2(K)) + 1e-6 * np.abs(want).max()
    assert (guard == 7.0).all()


def test_gemm_rejects_bad_k(stream):
    a = torch.zeros(64, dtype=torch.float16, device="cuda")
    with pytest.raises(P.CtnError):
        B.op_gemm(a, a, a, a, 2, 2, 12, P.EPI_BIAS_F16, stream)


def test_ops_reject_misaligned_operands(stream):
    """The kernels read rows in 16-byte pieces; an operand that starts elsewhere is refused on the host,
    before any launch."""
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    base = buf.data_ptr()
    assert base % 256 == 0
    ok = base + 4096
    for a, w, out in ((ok + 2, ok + 8192, ok + 16384), (ok, ok + 8192 + 8, ok + 16384), (ok, ok + 8192, ok + 16384 + 2)):
        with pytest.raises(P.CtnError) as e:
            B.op_gemm(a, w, base, out, 8, 16, 64, P.EPI_F32, stream)
        assert e.value.code == -1
    with pytest.raises(P.CtnError):
        B.op_layernorm(ok + 4, base, base, ok + 8192, 2, 128, stream)          # x off a 16-byte boundary
    with pytest.raises(P.CtnError):
        B.op_layernorm(ok, base + 2, base, ok + 8192, 2, 128, stream)          # gain off an 8-byte boundary
    with pytest.raises(P.CtnError):
        B.op_attention(ok + 8, ok + 32768, 1, 4, 1, 64, stream)
    with pytest.raises(P.CtnError):
        B.op_embed(base, ok + 2, ok + 8192, ok + 16384, 2, 2, 64, 8, 0, stream)
    stream.synchronize()
    assert int(buf.max()) == 0                                                 # nothing ran


@pytest.mark.parametrize("batch,seq,heads,d", [(1, 8, 12, 64), (2, 33, 3, 64), (4, 256, 16, 128), (1, 64, 16, 128),
                                               (2, 129, 2, 128), (16, 128, 10, 128), (1, 300, 2, 64),
                                               (1, 2048, 1, 64), (1, 1, 1, 128), (3, 127, 5, 64),
                                               (8, 256, 16, 128), (4, 200, 40, 64)])   # (256 and more wide workgroups)
def test_attention(stream, batch, seq, heads, d):
    rng = np.random.default_rng(batch * seq + heads + d)
    hl = heads * d
    qkv = f16(rng, (batch * seq, 3 * hl), 1.5)
    q, k, v = (qkv[:, i * hl:(i + 1) * hl].astype(np.float64).reshape(batch, seq, hl) for i in range(3))
    want = O.attention(q, k, v, heads).reshape(batch * seq, hl)
    out = torch.full((batch * seq, hl), float("nan"), dtype=torch.float16, device="cuda")
    B.op_attention(dev(qkv), out, batch, seq, heads, d, stream)
    stream.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    # probabilities are rounded to fp16 before the second product, outputs to fp16
    assert np.abs(got - want).max() <= 4e-3 * max(1.0, np.abs(want).max())
    assert np.abs(got - want).mean() <= 4e-4 * np.abs(want).mean() + 1e-5


@pytest.mark.parametrize("cfg", range(18))
@pytest.mark.parametrize("M,N,K,epi", [(300, 520, 328, P.EPI_BIAS_RESID_F32), (257, 129, 64, P.EPI_BIAS_RELU_F16),
                                       (61, 200, 1096, P.EPI_BIAS_F16), (9, 77, 40, P.EPI_F32),
                                       (300, 520, 320, P.EPI_BIAS_F16)])
def test_gemm_every_tile_configuration(stream, cfg, M, N, K, epi):
    """Each tile shape the library can pick, forced through the tuning hook, on ragged sizes."""
    hooks = Hooks()
    rng = np.random.default_rng(cfg * 1000 + M)
    A, W, bias = f16(rng, (M, K)), f16(rng, (N, K), 0.05), f16(rng, N, 0.5)
    res = rng.standard_normal((M, N)).astype(np.float32)
    acc = A.astype(np.float64) @ W.astype(np.float64).T + bias.astype(np.float64)
    if epi == P.EPI_BIAS_RESID_F32:
        want, out = res + acc, dev(res)
    elif epi == P.EPI_BIAS_RELU_F16:
        want, out = np.maximum(acc, 0), torch.empty(M, N, dtype=torch.float16, device="cuda")
    elif epi == P.EPI_BIAS_F16:
        want, out = acc, torch.empty(M, N, dtype=torch.float16, device="cuda")
    else:
        want, out = acc - bias.astype(np.float64), torch.empty(M, N, dtype=torch.float32, device="cuda")
    hooks.set(cfg)
    try:
        hooks.gemm(dev(A), dev(W), dev(bias), out, M, N, K, epi, stream)
        stream.synchronize()
    finally:
        hooks.set(-1)
    got = out.cpu().numpy().astype(np.float64)
    tol = 2.0 ** -10 * np.abs(want) + 1e-4 if out.dtype == torch.float16 else 1e-4
    assert np.all(np.abs(got - want) <= tol)
    for bad in (18, -2, 99, 110):      # 100..109 are the fill / load-depth / hand-over / reduction / tail switches, nothing else is accepted
        with pytest.raises(P.CtnError) as e:
            B.test_op_gemm(dev(A), dev(W), dev(bias), out, M, N, K, epi, None, [cfg, bad], stream)
        assert e.value.code == -1


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4, 5, 6, 7, 11, 12, 13, 14, 15, 17])
@pytest.mark.parametrize("M,N,K,epi", [(300, 520, 320, P.EPI_BIAS_RESID_F32), (257, 129, 64, P.EPI_BIAS_RELU_F16),
                                       (640, 1100, 1088, P.EPI_BIAS_F16), (64, 264, 2048, P.EPI_F32)])
def test_gemm_loads_two_steps_ahead_change_nothing(stream, cfg, M, N, K, epi):
    """The register-staged tiles with a second stage of global loads in flight (K a multiple of the tile's
    K step: one, two, five, seventeen steps; ragged edges; K slices with the workspace) against the plain loop:
    same K order, so the same bits."""
    hooks = Hooks()
    rng = np.random.default_rng(cfg * 77 + M + K)
    A, W, bias = f16(rng, (M, K)), f16(rng, (N, K), 0.05), f16(rng, N, 0.5)
    res = rng.standard_normal((M, N)).astype(np.float32)
    dA, dW, db = dev(A), dev(W), dev(bias)
    ws = torch.full((16 * M * N + 64,), float("nan"), dtype=torch.float32, device="cuda")
    outs = {}
    try:
        hooks.set(100)                       # (direct fills off, so that configuration 0 is register staged too)
        hooks.set(cfg)
        for hook in (103, 102):
            hooks.set(hook)
            out = dev(res) if epi in (P.EPI_BIAS_RESID_F32, P.EPI_F32) else torch.empty(M, N, dtype=torch.float16, device="cuda")
            guard = torch.full((4096,), 7.0, dtype=torch.float32, device="cuda")
            hooks.gemm(dA, dW, db, out, M, N, K, epi, stream, ws)
            stream.synchronize()
            assert (guard == 7.0).all()
            outs[hook] = out.cpu().numpy()
    finally:
        hooks.set(103)
        hooks.set(101)
        hooks.set(-1)
    assert np.array_equal(outs[103], outs[102])
    acc = A.astype(np.float64) @ W.astype(np.float64).T
    want = {P.EPI_BIAS_F16: acc + bias.astype(np.float64), P.EPI_BIAS_RELU_F16: np.maximum(acc + bias.astype(np.float64), 0),
            P.EPI_BIAS_RESID_F32: res + acc + bias.astype(np.float64), P.EPI_F32: acc}[epi]
    got, scale = outs[103].astype(np.float64), np.sqrt(K) * 0.05
    if outs[103].dtype == np.float16:
        assert np.all(np.abs(got - want) <= 2.0 ** -10 * np.abs(want) + 1e-4 * scale + 1e-7)
    else:
        assert np.abs(got - want).max() <= 2e-5 * scale * max(1.0, np.log2(K)) + 1e-6 * np.abs(want).max()


@pytest.mark.parametrize("M,N,K", [(1024, 2048, 512), (1000, 1100, 192), (129, 257, 64), (2048, 1280, 1280), (1024, 4096, 8192)])
@pytest.mark.parametrize("epi", [P.EPI_BIAS_F16, P.EPI_BIAS_RELU_F16, P.EPI_BIAS_RESID_F32, P.EPI_F32])
def test_gemm_direct_lds_fill_equals_register_staged(stream, M, N, K, epi):
    """128x128x64 tiles filled straight from global memory into LDS (K a multiple of 64) against the same
    tiles staged through registers: same K order, so the same bits; ragged edges, an odd number of K steps,
    one-step products and (with the workspace, last shape) K slices included."""
    hooks = Hooks()
    rng = np.random.default_rng(M + 5 * N + K + epi)
    A, W, bias = f16(rng, (M, K)), f16(rng, (N, K), 0.05), f16(rng, N, 0.5)
    res = rng.standard_normal((M, N)).astype(np.float32)
    dA, dW, db = dev(A), dev(W), dev(bias)
    ws = torch.full((4 * M * N + 64,), float("nan"), dtype=torch.float32, device="cuda")
    outs = {}
    try:
        for cfg in (0, 17):
            hooks.set(cfg)
            out = dev(res) if epi in (P.EPI_BIAS_RESID_F32, P.EPI_F32) else torch.empty(M, N, dtype=torch.float16, device="cuda")
            guard = torch.full((4096,), 7.0, dtype=torch.float32, device="cuda")
            hooks.gemm(dA, dW, db, out, M, N, K, epi, stream)
            stream.synchronize()
            assert (guard == 7.0).all()
            outs[cfg] = out.cpu().numpy()
        hooks.set(-1)          # the library's own choice with a workspace (K slices at M = 1024, K = 8192)
        for hook in (101, 100):
            hooks.set(hook)
            out = dev(res) if epi in (P.EPI_BIAS_RESID_F32, P.EPI_F32) else torch.empty(M, N, dtype=torch.float16, device="cuda")
            hooks.gemm(dA, dW, db, out, M, N, K, epi, stream, ws)
            stream.synchronize()
            outs[hook] = out.cpu().numpy()
    finally:
        hooks.set(101)
        hooks.set(-1)
    assert np.array_equal(outs[0], outs[17])
    assert np.array_equal(outs[101], outs[100])
    acc = A.astype(np.float64) @ W.astype(np.float64).T
    want = {P.EPI_BIAS_F16: acc + bias.astype(np.float64), P.EPI_BIAS_RELU_F16: np.maximum(acc + bias.astype(np.float64), 0),
            P.EPI_BIAS_RESID_F32: res + acc + bias.astype(np.float64), P.EPI_F32: acc}[epi]
    got, scale = outs[0].astype(np.float64), np.sqrt(K) * 0.05
    if outs[0].dtype == np.float16:
        assert np.all(np.abs(got - want) <= 2.0 ** -10 * np.abs(want) + 1e-4 * scale + 1e-7)
    else:
        assert np.abs(got - want).max() <= 2e-5 * scale * max(1.0, np.log2(K)) + 1e-6 * np.abs(want).max()


@pytest.mark.parametrize("M,N,K", [(1024, 8832, 2048), (2048, 5120, 2048), (1000, 8744, 2112)])
@pytest.mark.parametrize("epi", [P.EPI_BIAS_F16, P.EPI_BIAS_RELU_F16, P.EPI_BIAS_RESID_F32, P.EPI_F32])
def test_gemm_tail_columns_in_k_slices(stream, M, N, K, epi):
    """A product whose 128x128 tiles end in a thinly filled round (552, 640 and 552 tiles against 512 slots): the
    columns of that round are computed in K slices by a second launch and added in a fixed order.  Same bar as
    any other product, the same bits when repeated, nothing written past the output, and close to the
    one-launch result (only the order of the fp32 additions differs in the tail columns)."""
    hooks = Hooks()
    rng = np.random.default_rng(M + 3 * N + K + epi)
    A, W, bias = f16(rng, (M, K)), f16(rng, (N, K), 0.05), f16(rng, N, 0.5)
    res = rng.standard_normal((M, N)).astype(np.float32)
    dA, dW, db = dev(A), dev(W), dev(bias)
    ws = torch.full((4 * M * 4096 + 64,), float("nan"), dtype=torch.float32, device="cuda")
    outs = []
    try:
        for hook in (109, 109, 108):
            hooks.set(hook)
            out = dev(res) if epi in (P.EPI_BIAS_RESID_F32, P.EPI_F32) else torch.empty(M, N, dtype=torch.float16, device="cuda")
            guard = torch.full((4096,), 7.0, dtype=torch.float32, device="cuda")
            hooks.gemm(dA, dW, db, out, M, N, K, epi, stream, ws)
            stream.synchronize()
            assert (guard == 7.0).all()
            outs.append(out.cpu().numpy())
    finally:
        hooks.set(109)
    assert np.array_equal(outs[0], outs[1])
    acc = A.astype(np.float64) @ W.astype(np.float64).T
    want = {P.EPI_BIAS_F16: acc + bias.astype(np.float64), P.EPI_BIAS_RELU_F16: np.maximum(acc + bias.astype(np.float64), 0),
            P.EPI_BIAS_RESID_F32: res + acc + bias.astype(np.float64), P.EPI_F32: acc}[epi]
    scale = np.sqrt(K) * 0.05
    for got in (outs[0].astype(np.float64), outs[2].astype(np.float64)):
        if outs[0].dtype == np.float16:
            assert np.all(np.abs(got - want) <= 2.0 ** -10 * np.abs(want) + 1e-4 * scale + 1e-7)
        else:
            assert np.abs(got - want).max() <= 2e-5 * scale * max(1.0, np.log2(K)) + 1e-6 * np.abs(want).max()
    n_main = (((M + 127) // 128) * ((N + 127) // 128)) // 512 * 512 // ((M + 127) // 128) * 128
    assert np.array_equal(outs[0][:, :n_main], outs[2][:, :n_main])      # the full rounds' columns: one launch either way


@pytest.mark.parametrize("M,N,K", [(64, 4096, 8192), (64, 520, 1096), (17, 6144, 4096), (33, 200, 264), (48, 8192, 512)])
@pytest.mark.parametrize("epi", [P.EPI_BIAS_F16, P.EPI_BIAS_RELU_F16, P.EPI_BIAS_RESID_F32, P.EPI_F32])
@pytest.mark.parametrize("force", [-1, 14, 15])
def test_gemm_split_k_with_workspace(stream, M, N, K, epi, force):
    """Small-M products with a scratch buffer: K split across workgroups, partials added in order;
    same bar as the one-pass product, and bit-identical when repeated."""
    hooks = Hooks()
    rng = np.random.default_rng(M + N + K + epi)
    A, W, bias = f16(rng, (M, K)), f16(rng, (N, K), 0.05), f16(rng, N, 0.5)
    res = rng.standard_normal((M, N)).astype(np.float32)
    acc = A.astype(np.float64) @ W.astype(np.float64).T
    if epi == P.EPI_BIAS_F16:
        want, mk = acc + bias.astype(np.float64), lambda: torch.empty(M, N, dtype=torch.float16, device="cuda")
    elif epi == P.EPI_BIAS_RELU_F16:
        want, mk = np.maximum(acc + bias.astype(np.float64), 0), lambda: torch.empty(M, N, dtype=torch.float16, device="cuda")
    elif epi == P.EPI_BIAS_RESID_F32:
        want, mk = res + acc + bias.astype(np.float64), lambda: dev(res)
    else:
        want, mk = acc, lambda: torch.empty(M, N, dtype=torch.float32, device="cuda")
    ws = torch.full((16 * M * N + 64,), float("nan"), dtype=torch.float32, device="cuda")
    outs = []
    hooks.set(force)
    try:
        for hook in (107, 107, 106):       # the reduction four columns at a time, again, then one column at a time
            hooks.set(hook)
            out = mk()
            hooks.gemm(dev(A), dev(W), dev(bias), out, M, N, K, epi, stream, ws)
            stream.synchronize()
            outs.append(out.cpu().numpy())
    finally:
        hooks.set(107)
        hooks.set(-1)
    assert np.array_equal(outs[0], outs[1])
    assert np.array_equal(outs[0], outs[2])       # both reductions add the slices in the same order
    got = outs[0].astype(np.float64)
    scale = np.sqrt(K) * 0.05
    if outs[0].dtype == np.float16:
        assert np.all(np.abs(got - want) <= 2.0 ** -10 * np.abs(want) + 1e-4 * scale + 1e-7)
    else:
        assert np.abs(got - want).max() <= 2e-5 * scale * max(1.0, np.log2(K)) + 1e-6 * np.abs(want).max()
