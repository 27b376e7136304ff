"""GPU check of newton_schulz_static_scratch, the entry point for callers that cannot
allocate: its output must equal newton_schulz's bit for bit when both use the same chunking,
and match the oracle to the Newton-Schulz tolerance, on two calls in a row that share the
library's one scratch buffer, the second on a smaller input."""
import pytest
import torch

import paper_2505_23725_amd as mlc
import synth_inputs as S
from oracle import muon
from helpers import NS_TOL, assert_ns_close, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(x_cpu):
    cnt, m, n = x_cpu.shape
    x = x_cpu.to(DEV)
    # the existing entry point with a work space of the built-in buffer's size: same chunking
    ws = torch.empty(min(mlc.STATIC_SCRATCH_BYTES, mlc.newton_schulz_workspace_bytes(cnt, m, n)),
                     dtype=torch.uint8, device=DEV)
    ref = torch.empty_like(x)
    mlc.newton_schulz(x, ref, ws)
    out = torch.empty_like(x)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    mlc.newton_schulz_static_scratch(x, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return ref.cpu(), out.cpu()


def test_two_calls_in_a_row_second_smaller():
    # first call: 40 matrices of 768 x 768 fill the 64 MiB buffer several times over (chunks);
    # second call: fewer and smaller matrices, ragged, through the same buffer
    big = S.normal((40, 768, 768), S.GRAD_STD, seed=11, stream=0, dtype=torch.bfloat16)
    small = S.normal((3, 200, 136), S.GRAD_STD, seed=11, stream=1, dtype=torch.float32)
    for x in (big, small):
        ref, out = _both(x)
        assert torch.equal(ref.view(torch.int32 if x.dtype == torch.float32 else torch.int16),
                           out.view(torch.int32 if x.dtype == torch.float32 else torch.int16))
        for i in (0, x.shape[0] - 1):
            assert_ns_close(to_f64(out[i]), muon.newton_schulz(to_f64(x[i]), 5), f"{tuple(x.shape)} matrix {i}")


def test_one_workgroup_chain_and_largest_shape():
    # 128 x 512 runs the one-launch chain; 2048 x 2048 is the largest square the buffer holds
    for shape, seed in (((5, 128, 512), 12), ((2, 2048, 2048), 13)):
        x = S.normal(shape, S.GRAD_STD, seed=seed, stream=0, dtype=torch.bfloat16)
        ref, out = _both(x)
        assert torch.equal(ref.view(torch.int16), out.view(torch.int16))
    assert_ns_close(to_f64(out[1]), muon.newton_schulz(to_f64(x[1]), 5), "2048 x 2048")


def test_too_large_is_refused_and_leaves_output_alone():
    x = torch.zeros(1, 2048, 8192, dtype=torch.bfloat16, device=DEV)
    out = torch.full_like(x, 3.0)
    with pytest.raises(mlc.MulocoError) as e:
        mlc.newton_schulz_static_scratch(x, out)
    assert e.value.code == -8
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())
