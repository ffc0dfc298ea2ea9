"""The entry point that allocates nothing: ctn_op_gemm_static takes the split-K scratch from the library's
static device array.  Its output must equal ctn_op_gemm_ws (caller's workspace of the same size) bit for
bit, on two calls in a row, the second with a smaller input that leaves stale partial tiles of the first
in the array."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
import paper_2306_13835_amd as P
from paper_2306_13835_amd import binding as B

pytestmark = pytest.mark.gpu


def f16(rng, shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float16)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_both(stream, ws, M, N, K, epi, seed):
    rng = np.random.default_rng(seed)
    A, W, bias = f16(rng, (M, K)), f16(rng, (N, K), 0.05), f16(rng, N, 0.5)
    res = rng.standard_normal((M, N)).astype(np.float32)
    dA, dW, db = dev(A), dev(W), dev(bias)

    def fresh():
        if epi in (P.EPI_BIAS_RESID_F32, P.EPI_F32):
            return dev(res)
        return torch.zeros(M, N, dtype=torch.float16, device="cuda")
    want_out, got_out = fresh(), fresh()
    torch.cuda.synchronize()
    B.op_gemm_ws(dA, dW, db, want_out, M, N, K, epi, ws, stream)
    B.op_gemm_static(dA, dW, db, got_out, M, N, K, epi, stream)
    stream.synchronize()
    want, got = want_out.cpu().numpy(), got_out.cpu().numpy()
    # the existing entry point itself against the definition (fp64), so that "equal" means "right"
    acc = A.astype(np.float64) @ W.astype(np.float64).T
    ref = {P.EPI_BIAS_F16: acc + bias.astype(np.float64), P.EPI_BIAS_RELU_F16: np.maximum(acc + bias.astype(np.float64), 0),
           P.EPI_BIAS_RESID_F32: res + acc + bias.astype(np.float64), P.EPI_F32: acc}[epi]
    scale = np.sqrt(K) * 0.05
    if want.dtype == np.float16:
        assert np.all(np.abs(want.astype(np.float64) - ref) <= 2.0 ** -10 * np.abs(ref) + 1e-4 * scale + 1e-7)
    else:
        assert np.abs(want - ref).max() <= 2e-5 * scale * max(1.0, np.log2(K)) + 1e-6 * np.abs(ref).max()
    return want, got


# (first call, second and smaller call): K-sliced 64x64 tiles, 32x128 tiles, 128x128 tiles in two to four
# slices with a ragged edge, and a shape that is never split
PAIRS = [((64, 4096, 8192), (33, 520, 1096)),
         ((24, 6144, 4096), (17, 200, 264)),
         ((1000, 1100, 4096), (130, 2048, 2048)),
         ((256, 2048, 2048), (8, 512, 4096))]


@pytest.mark.parametrize("first,second", PAIRS)
@pytest.mark.parametrize("epi", [P.EPI_BIAS_F16, P.EPI_BIAS_RELU_F16, P.EPI_BIAS_RESID_F32, P.EPI_F32])
def test_static_scratch_product_equals_workspace_product(first, second, epi):
    stream = torch.cuda.Stream()
    n_ws = B.static_scratch_bytes() // 4
    assert n_ws * 4 == 64 << 20
    ws = torch.full((n_ws,), float("nan"), dtype=torch.float32, device="cuda")
    for k, (M, N, K) in enumerate((first, second)):
        want, got = run_both(stream, ws, M, N, K, epi, seed=1000 * k + M + N + K + epi)
        assert np.array_equal(want, got), (M, N, K, epi)


def test_static_scratch_rejects_what_does_not_fit():
    stream = torch.cuda.Stream()
    a = torch.zeros(16, dtype=torch.float16, device="cuda")
    L = P.lib()
    # 16 slices of 256 x 8192 fp32 = 128 MiB; 4 slices of 4096 x 4096 fp32 = 256 MiB
    for M, N in ((256, 8192), (4096, 4096)):
        rc = L.ctn_op_gemm_static(a.data_ptr(), a.data_ptr(), a.data_ptr(), a.data_ptr(), M, N, 64, P.EPI_F32,
                                  stream.cuda_stream)
        assert rc == -2, (M, N, rc)           # CTN_E_TOO_BIG, nothing launched
    assert L.ctn_op_gemm_static(None, a.data_ptr(), a.data_ptr(), a.data_ptr(), 8, 8, 64, P.EPI_F32,
                                stream.cuda_stream) == -1
    stream.synchronize()
