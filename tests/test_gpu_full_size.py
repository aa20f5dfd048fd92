"""Config 3 at its full size (32 layers, d_model 4096, vocabulary 126 464), in the launch configuration the
benchmark times: the stage-1 call (1 x 512 tokens) and the verification call (4 drafts x 512 tokens) against
the fp64 oracle over the full depth.  At this width the logit tolerance is calibrated by the oracle itself
(see _compare in test_gpu_forward.py): no bf16 evaluation of this network stays within 2e-2 of exact arithmetic.  The oracle needs about 12 s per
sequence-forward on 16 host cores and the fp32 host copy of the weights about 32 GB, so the verification batch
is compared on its first and last draft only (sampled outputs; every draft runs through the same kernels)."""
import time

import numpy as np
import pytest
import torch

import psd_inputs as inp
from oracle import psd_oracle as orc

pytestmark = pytest.mark.gpu


def test_config3_full_depth_stage1_and_verify():
    import psutil
    if psutil.virtual_memory().available < 60 * 2 ** 30:
        pytest.skip("needs about 40 GB of free host memory for the fp32 host copy of an 8B-parameter model")
    import paper_2605_15609_amd as psd
    from tests.gpu_common import say
    from tests.test_gpu_forward import _compare
    w = inp.WORKLOADS[3]
    shape, N, P, L, K = w.shape, w.seq_len, w.prompt_len, w.block_len, w.n_drafts
    t0 = time.perf_counter()
    host = inp.draw_model(shape, N, threads=16)
    say(f"[full-size] host model drawn in {time.perf_counter() - t0:.0f} s")
    model = psd.Model.from_host(host)
    say(f"[full-size] uploaded after {time.perf_counter() - t0:.0f} s")
    tokens = inp.initial_state(w)[0]
    _compare(model, host, [tokens], P, L, 2e-2, "cfg3-full/stage-1", calibrate=True)
    say(f"[full-size] stage-1 compared after {time.perf_counter() - t0:.0f} s")
    # drafts from the oracle's own stage-1 decisions (Eq. 1, Eq. 2), then the batched verification call
    top1, conf = orc.forward_confidence(host, tokens, P, L)
    policy, graph = orc.Policy(w.tau, w.k_min, w.k_max), orc.chain_graph(K)
    committed, _ = orc.select_unmask(tokens, P, L, top1, conf, policy, shape.mask_id)
    sigma, m, drafts = orc.build_drafts(committed, P, L, top1, conf, graph, shape.mask_id)
    assert m >= K - 1, "the first block leaves enough masks for every draft to differ"
    say(f"[full-size] drafts built after {time.perf_counter() - t0:.0f} s")
    _compare(model, host, [np.asarray(d, dtype=np.int32) for d in drafts], P, L, 2e-2, "cfg3-full/verify", check=(0, K - 1), calibrate=True)
    say(f"[full-size] verification compared after {time.perf_counter() - t0:.0f} s")
    model.close()
    del host
