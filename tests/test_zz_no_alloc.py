"""The allocation-free column-sum entry point (partial sums in a device array built into the
library) against the workspace-taking entry point it is a variant of, and against the plain
definition: two calls in a row on one stream, the second on a smaller input, so that stale
partial sums of the first call would show."""
import numpy as np
import pytest
import torch

from oracle import stage_oracle as O
from paper_2111_04007_amd import binding as B
from paper_2111_04007_amd.synth import to_f64

pytestmark = pytest.mark.gpu

DT = {"f32": torch.float32, "bf16": torch.bfloat16}


def _rnd(shape, dtype, seed):
    g = np.random.Generator(np.random.Philox(key=[seed, 77]))
    return torch.from_numpy(g.standard_normal(shape)).to(DT[dtype]).cuda()


def _both(a):
    rows, n = a.shape
    want = torch.full((n,), 0.5, dtype=torch.float32, device="cuda")
    partial = torch.empty(B.colreduce_scratch_bytes(rows, n) // 4, dtype=torch.float32, device="cuda")
    B.op_colsum(a, want, partial)
    got = torch.full((n,), 0.5, dtype=torch.float32, device="cuda")
    B.op_colsum_static(a, got)
    return got, want


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_colsum_static_matches_workspace_variant_on_two_calls(dtype):
    big = _rnd((2048, 4096), dtype, 31)       # 8 row chunks of partial sums, 128 KiB of scratch
    small = _rnd((300, 72), dtype, 32)        # ragged rows and columns, a corner of the same scratch
    got_big, want_big = _both(big)
    got_small, want_small = _both(small)
    torch.cuda.synchronize()
    for got, want, a in ((got_big, want_big, big), (got_small, want_small, small)):
        assert torch.equal(got, want)          # same kernels, same order of additions: bit-identical
        assert O.rel_l2(to_f64(got), 0.5 + to_f64(a).sum(axis=0)) <= 1e-5


def test_colsum_static_rejects_oversized_shapes_without_touching_the_gpu():
    cap = B.colsum_static_max_bytes()
    assert cap == 4 << 20
    rows, n = 256 * 64, 32768                  # 64 chunks x 32768 columns x 4 B = 8 MiB of partial sums
    assert B.colreduce_scratch_bytes(rows, n) > cap
    a = torch.empty((1, 8), dtype=torch.bfloat16, device="cuda")   # never read: the size check comes first
    out = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(B.VarunaError) as ei:
        B.load().varuna_op_colsum_static  # symbol exists
        B._check(B.load().varuna_op_colsum_static(B.BF16, rows, n, B._ptr(a), B._ptr(out), B._stream_ptr()))
    assert ei.value.code == B.EUNSUPPORTED
