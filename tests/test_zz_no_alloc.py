"""The entry point for callers that cannot allocate (GPU only): hydra_op_colsum_noalloc keeps its partial sums in
an array built into the library instead of caller scratch.  It runs the kernels of hydra_op_colsum, so its output
must equal that entry point's bit for bit: on two calls in a row, the second on a smaller input (the array keeps the
first call's contents), in both operand types, with a group of problems; requests beyond the array are refused."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "GPU tests need a HIP device"
    return t


@pytest.fixture(scope="module")
def ops():
    from paper_2107_06469_amd import ops as o
    return o


def _case(torch, ops, dtype, M, N, G, seed):
    r = np.random.default_rng(seed)
    ld = (N + 7) // 8 * 8
    srcs, want, got = [], [], []
    for g in range(G):
        h = np.zeros((M, ld), dtype=np.float32)
        h[:, :N] = r.normal(size=(M, N))
        t = torch.from_numpy(h).cuda()
        srcs.append(t.to(torch.bfloat16) if dtype == 1 else t)
        want.append(torch.full((N,), -1.0, dtype=torch.float32, device="cuda"))
        got.append(torch.full((N,), -2.0, dtype=torch.float32, device="cuda"))
    parts = [torch.zeros(max(1, ops.hydra_op_colsum_part_floats(M, N)), dtype=torch.float32, device="cuda") for _ in range(G)]
    ops.hydra_op_colsum(dtype, M, N, ld, srcs, want, parts)
    ops.hydra_op_colsum_noalloc(dtype, M, N, ld, srcs, got)
    torch.cuda.synchronize()
    for g in range(G):
        a, b = got[g].cpu().numpy(), want[g].cpu().numpy()
        assert np.array_equal(a, b), (dtype, M, N, g, float(np.abs(a - b).max()))
        # and both are the column sums (fp64 sum of the values the kernel read)
        ref = srcs[g].float().cpu().numpy().astype(np.float64)[:, :N].sum(axis=0)
        assert np.allclose(a, ref, rtol=0, atol=2 * M * 2.0 ** -24 * 4)


@pytest.mark.parametrize("dtype", [0, 1])
def test_two_calls_in_a_row_the_second_smaller(torch, ops, dtype):
    _case(torch, ops, dtype, 5000, 1000, 3, seed=1)     # 20 chunks of 256 rows, ragged last chunk
    _case(torch, ops, dtype, 777, 130, 2, seed=2)       # smaller: reads only what it wrote itself
    _case(torch, ops, dtype, 97, 10, 1, seed=3)         # one chunk: no partial sums at all


def test_requests_beyond_the_built_in_array_are_refused(torch, ops):
    from paper_2107_06469_amd.hydra import HydraError
    cap = ops.hydra_op_colsum_noalloc_max_floats()
    assert cap == 1 << 20
    M, N = 256 * 64 + 1, 8192                           # 65 chunks x 8192 columns x 2 problems > 2^20 floats
    assert 2 * ops.hydra_op_colsum_part_floats(M, N) > cap
    x = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(HydraError) as e:
        ops.hydra_op_colsum_noalloc(0, M, N, N, [x, x], [x, x])
    assert e.value.status == 1 and "scratch" in str(e.value)
    M, N = 256 * 64, 8192                               # exactly the capacity with two problems
    assert 2 * ops.hydra_op_colsum_part_floats(M, N) == cap
    src = [torch.ones((M, N), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    out = [torch.zeros(N, dtype=torch.float32, device="cuda") for _ in range(2)]
    ops.hydra_op_colsum_noalloc(1, M, N, N, src, out)
    torch.cuda.synchronize()
    assert all(bool((o == float(M)).all()) for o in out)
