"""The LM-head confidence pass through the entry point that allocates nothing (its partial results live in a
static device array of the library) against the same pass with a caller-provided scratch buffer: identical kernels,
so the outputs must be bit-identical -- on two calls in a row, the second on a smaller input, so that whatever the
first call left in the shared array is seen not to leak into the second."""
import numpy as np
import pytest
import torch

import psd_inputs as inp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(rows, V, d, seed):
    rng = np.random.default_rng(seed)
    y = inp.round_to_bf16(rng.standard_normal((rows, d), dtype=np.float32))
    W = inp.round_to_bf16(rng.standard_normal((V, d), dtype=np.float32) * 0.02)
    to = lambda a: torch.from_numpy(a).to(DEV).to(torch.bfloat16)
    return to(y), to(W)


def test_static_scratch_head_equals_the_caller_scratch_head_twice_in_a_row():
    from paper_2605_15609_amd import binding as B
    scale = 1.3
    for rows, V, d, seed in ((128, 32000, 512, 1), (37, 5000, 512, 2), (192, 9000, 576, 3), (1, 3001, 64, 4)):
        print(f"[no-alloc] rows={rows} V={V} d={d}", flush=True)
        y, W = _case(rows, V, d, seed)
        Wp, yp = B.kernel_pack_rows(W), B.kernel_pack_rows(y)
        want_sum, want_arg = B.kernel_head_stream_bf16(y, Wp, V, scale, V - 1, y_packed=yp)
        got_sum = torch.full((rows,), -7.0, dtype=torch.float32, device=DEV)
        got_arg = torch.full((rows,), -7, dtype=torch.int32, device=DEV)
        B.kernel_head_stream_static_bf16(yp, Wp, rows, V, d, scale, V - 1, got_sum, got_arg)
        torch.cuda.synchronize()
        assert torch.equal(got_arg, want_arg), (rows, V)
        assert torch.equal(got_sum, want_sum), (rows, V)
        assert bool((got_arg >= 0).all()) and bool((got_arg < V - 1).all()) and bool((got_sum >= 1.0).all())


def test_static_scratch_head_rejects_what_the_array_cannot_hold():
    from paper_2605_15609_amd import binding as B
    y, W = _case(8, 3001, 64, 5)
    Wp, yp = B.kernel_pack_rows(W), B.kernel_pack_rows(y)
    out_sum = torch.zeros((8,), dtype=torch.float32, device=DEV)
    out_arg = torch.zeros((8,), dtype=torch.int32, device=DEV)
    with pytest.raises(B.PsdError, match="static scratch"):
        B.kernel_head_stream_static_bf16(yp, Wp, 8, 163841, 64, 1.0, 5, out_sum, out_arg)     # vocabulary beyond the limit
    with pytest.raises(B.PsdError):
        B.kernel_head_stream_static_bf16(yp, Wp, 193, 3001, 64, 1.0, 5, out_sum, out_arg)      # rows beyond the limit
