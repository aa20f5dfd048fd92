"""The C-ABI library loads and exports every symbol that include/psd.h declares (CPU only)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2605_15609_amd as psd
    if not os.path.exists(psd.library_path()):
        from paper_2605_15609_amd import build
        build.build()
    return psd.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "psd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(psd_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"psd_forward_confidence", "psd_select_unmask", "psd_build_drafts", "psd_verify_accept",
            "psd_decode_block"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_structure_layouts_agree_with_the_binding(lib):
    from paper_2605_15609_amd import binding as B
    n = lib.psd_struct_sizes(None, 0)
    got = (ctypes.c_int32 * n)()
    assert lib.psd_struct_sizes(got, n) == n == 8
    assert list(got) == [ctypes.sizeof(t) for t in (B._Config, B._Weights, B._Policy, B._Graph, B._Stats, B._Work, B._GraphScore,
                                                    B._DebugLayout)]
    assert got[2] == 24 and got[6] == 40           # psd_policy: float + 5 x int32; psd_graph_score: 3 doubles + 2 x int64


def test_host_only_entry_points(lib):
    import paper_2605_15609_amd as psd
    assert lib.psd_status_string(0) == b"ok" and lib.psd_status_string(-3).startswith(b"workspace")
    g = psd.chain_graph(4)
    assert g.rank_sets == (0, 1, 3, 7)
    assert psd.chain_graph(3, 2).rank_sets == (0, 3, 15)
    with pytest.raises(psd.PsdError):
        psd.chain_graph(40)
    # subset lattice: every subset of the top ranks exactly once, root first, by size
    import itertools
    for depth in range(0, 6):
        sets = psd.lattice_graph(depth).rank_sets
        want = [sum(1 << r for r in c) for n in range(depth + 1) for c in itertools.combinations(range(depth), n)]
        assert sorted(sets) == sorted(want) and len(sets) == 2 ** depth and sets[0] == 0
        assert [bin(x).count("1") for x in sets] == sorted(bin(x).count("1") for x in sets)
    with pytest.raises(psd.PsdError):
        psd.lattice_graph(6)
    assert lib.psd_decode_scratch_bytes(1, 512, 32, 4) > 4 * 512 * 4
    assert lib.psd_decode_scratch_bytes(0, 512, 32, 4) < 0


def test_workspace_and_work_accounting(lib):
    import psd_inputs as inp
    from paper_2605_15609_amd.binding import _Config, _Work
    s = inp.WORKLOADS[3].shape
    cfg = _Config(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.d_head, s.d_ffn, s.vocab, s.mask_id, s.rms_eps, 0, 1,
                  1.0, 512)
    small = lib.psd_workspace_bytes(ctypes.byref(cfg), 1, 512, 32)
    big = lib.psd_workspace_bytes(ctypes.byref(cfg), 4, 512, 32)
    assert 0 < small < big < 2 ** 33
    w = _Work()
    assert lib.psd_forward_work(ctypes.byref(cfg), 4, 512, 32, ctypes.byref(w)) == 0
    # config 3 verify call: ~28.6 TFLOP of layer contractions, 1.036 GB LM-head weights
    assert abs(w.gemm_flops / 28.59e12 - 1) < 0.01
    assert abs(w.attn_flops / 0.55e12 - 1) < 0.01
    assert abs(w.head_bytes / 1.037e9 - 1) < 0.01
    bad = _Config(2, 100, 4, 4, 25, 256, 300, 299, 1e-5, 0, 1, 1.0, 64)
    assert lib.psd_workspace_bytes(ctypes.byref(bad), 1, 32, 8) < 0


def test_the_binding_rejects_tensors_the_library_would_misread(lib):
    """The library reads raw pointers: rotary tables handed over as bf16 would be read as fp32 (garbage, and past
    the end of the tensor).  Model checks dtype and extent of every tensor before psd_create."""
    import numpy as np
    import torch
    import psd_inputs as inp
    from paper_2605_15609_amd import binding as B
    shape = inp.cut_down(inp.WORKLOADS[2].shape, n_layers=1, vocab=512)
    host = inp.draw_model(shape, 64)

    def tensors(rope_dtype=torch.float32, max_seq=64):
        mat = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16)
        vec = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.float32)
        t = {"tok_emb": mat(host.tok_emb), "lm_head": mat(host.lm_head), "final_norm": vec(host.final_norm),
             "rope_cos": torch.from_numpy(host.rope_cos[:max_seq]).to(rope_dtype), "rope_sin": torch.from_numpy(host.rope_sin[:max_seq]).to(rope_dtype)}
        lt = {k: (None if v is None else (mat(v) if v.ndim == 2 else vec(v))) for k, v in host.layers[0].items()}
        B.pack_qkv(lt)
        return t, [lt]

    t, layers = tensors(rope_dtype=torch.bfloat16)
    with pytest.raises(B.PsdError, match="rope_cos"):
        B.Model(shape, 64, t, layers, device="cpu")
    t, layers = tensors(max_seq=32)                 # tables shorter than max_seq
    with pytest.raises(B.PsdError, match="rope_cos"):
        B.Model(shape, 64, t, layers, device="cpu")
    t, layers = tensors()
    layers[0]["wo"] = layers[0]["wo"].float()        # a matrix in the wrong dtype
    with pytest.raises(B.PsdError, match="layer 0 wo"):
        B.Model(shape, 64, t, layers, device="cpu")
