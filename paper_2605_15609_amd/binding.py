"""ctypes binding of libpsd.so: same call names as include/psd.h, torch tensors in and out.

Nothing here computes: tensors are allocated with torch, their device pointers and the
current HIP stream are handed to the library, and every step of the PSD path runs in its
kernels.  Loading fails loudly when the library has not been built; there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
MAX_NODES = 32
MAX_BLOCK = 64
HIST = MAX_NODES + MAX_BLOCK + 1


class PsdError(RuntimeError):
    pass


class _Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("d_head", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("mask_id", C.c_int32),
                ("rms_eps", C.c_float), ("qkv_bias", C.c_int32), ("dtype", C.c_int32), ("logit_scale", C.c_float),
                ("max_seq", C.c_int32), ("attention", C.c_int32)]


_PP = C.POINTER(C.c_void_p)


class _Weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p), ("rope_cos", C.c_void_p),
                ("rope_sin", C.c_void_p), ("attn_norm", _PP), ("wq", _PP), ("wk", _PP), ("wv", _PP), ("bq", _PP),
                ("bk", _PP), ("bv", _PP), ("wo", _PP), ("ffn_norm", _PP), ("w_gate", _PP), ("w_up", _PP), ("w_down", _PP),
                ("w_down_stride", C.c_int32)]


class _Policy(C.Structure):
    _fields_ = [("tau", C.c_float), ("k_min", C.c_int32), ("k_max", C.c_int32), ("eos_stop", C.c_int32),
                ("eos_id", C.c_int32), ("single_forward", C.c_int32)]


class _Graph(C.Structure):
    _fields_ = [("K", C.c_int32), ("rank_set", C.c_uint64 * MAX_NODES)]


class _Stats(C.Structure):
    _fields_ = [("invocations", C.c_int64), ("tokens_policy", C.c_int64), ("tokens_draft", C.c_int64),
                ("tokens_postverify", C.c_int64), ("depth_hist", C.c_int32 * HIST), ("tokens_counted", C.c_int64),
                ("stopped", C.c_int32), ("eos_pos", C.c_int32)]


class _GraphScore(C.Structure):
    _fields_ = [("seconds", C.c_double), ("tokens_per_s", C.c_double), ("tpf", C.c_double), ("tokens", C.c_int64),
                ("invocations", C.c_int64)]


class _Work(C.Structure):
    _fields_ = [("gemm_flops", C.c_double), ("attn_flops", C.c_double), ("head_flops", C.c_double),
                ("head_bytes", C.c_double), ("weight_bytes", C.c_double)]


class _DebugLayout(C.Structure):
    _fields_ = [("off_a", C.c_int64), ("off_qkv", C.c_int64), ("off_vt", C.c_int64), ("off_o", C.c_int64),
                ("off_act", C.c_int64), ("ld_qkv", C.c_int32), ("ld_act", C.c_int32), ("ld_vt", C.c_int32),
                ("reserved", C.c_int32)]


_lib = None


def library_path() -> str:
    return os.environ.get("PSD_LIBRARY", os.path.join(_HERE, "libpsd.so"))


def load_library():
    """Loads libpsd.so (built by paper_2605_15609_amd/build.py).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise PsdError(f"{path} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    sig = {
        "psd_status_string": (C.c_char_p, [i32]),
        "psd_last_error": (C.c_char_p, []),
        "psd_create": (i32, [C.POINTER(_Config), C.POINTER(_Weights), C.POINTER(vp)]),
        "psd_destroy": (i32, [vp]),
        "psd_debug_set_plain": (i32, [vp, i32]),
        "psd_debug_workspace_layout": (i32, [C.POINTER(_Config), i32, i32, i32, C.POINTER(_DebugLayout)]),
        "psd_debug_layer": (i32, [vp, i32, vp, i32, i32, i32, i32, vp, i64, vp]),
        "psd_workspace_bytes": (i64, [C.POINTER(_Config), i32, i32, i32]),
        "psd_decode_scratch_bytes": (i64, [i32, i32, i32, i32]),
        "psd_struct_sizes": (i32, [C.POINTER(i32), i32]),
        "psd_graph_chain": (i32, [i32, i32, C.POINTER(_Graph)]),
        "psd_graph_lattice": (i32, [i32, C.POINTER(_Graph)]),
        "psd_calibrate_graph": (i32, [vp, vp, vp, i32, i32, i32, i32, C.POINTER(_Policy), C.POINTER(_Graph), i32,
                                      C.POINTER(_GraphScore), C.POINTER(i32), vp, i32, vp, i64, vp]),
        "psd_forward_confidence": (i32, [vp, vp, i32, i32, i32, i32, vp, vp, vp, i64, vp]),
        "psd_forward_logits": (i32, [vp, vp, i32, i32, i32, i32, vp, vp, i64, vp]),
        "psd_select_unmask": (i32, [vp, vp, i32, i32, i32, i32, vp, vp, C.POINTER(_Policy), vp, vp, vp]),
        "psd_build_drafts": (i32, [vp, vp, i32, i32, i32, i32, vp, vp, C.POINTER(_Graph), vp, vp, vp, vp]),
        "psd_accept": (i32, [vp, vp, vp, i32, i32, i32, i32, vp, vp, C.POINTER(_Graph), C.POINTER(_Policy), vp, vp, vp,
                             vp, vp]),
        "psd_verify_accept": (i32, [vp, vp, vp, i32, i32, i32, i32, vp, vp, C.POINTER(_Graph), C.POINTER(_Policy), vp,
                                    vp, vp, vp, vp, i64, vp]),
        "psd_kv_cache_bytes": (i64, [C.POINTER(_Config), i32]),
        "psd_kv_reset": (i32, [vp, vp, i32, i32, vp]),
        "psd_kv_prefill": (i32, [vp, vp, i32, i32, i32, i32, vp, i32, vp, i64, vp]),
        "psd_forward_confidence_cached": (i32, [vp, vp, i32, i32, i32, i32, i32, vp, i32, vp, vp, vp, vp, i64, vp]),
        "psd_decode_block_cached": (i32, [vp, vp, i32, i32, i32, i32, C.POINTER(_Policy), C.POINTER(_Graph), C.POINTER(_Stats),
                                           vp, i32, vp, i64, vp]),
        "psd_decode_block": (i32, [vp, vp, i32, i32, C.POINTER(i32), i32, C.POINTER(_Policy), C.POINTER(_Graph), C.POINTER(_Stats),
                                   vp, i64, vp]),
        "psd_decode": (i32, [vp, vp, i32, i32, C.POINTER(i32), i32, C.POINTER(_Policy), C.POINTER(_Graph), C.POINTER(_Stats),
                             i32, C.POINTER(i32), vp, i64, vp]),
        "psd_forward_confidence_approx": (i32, [vp, vp, i32, i32, i32, i32, i32, i32, vp, i32, vp, vp, vp, vp, i64, vp]),
        "psd_decode_block_approx": (i32, [vp, vp, i32, i32, i32, i32, C.POINTER(_Policy), C.POINTER(_Graph), C.POINTER(_Stats),
                                          vp, i32, vp, i64, vp]),
        "psd_kernel_gemm_bf16": (i32, [vp, vp, vp, i64, i32, i32, i32, i32, i32, vp, vp, vp, i32, vp]),
        "psd_kernel_gemm_residual_splitk": (i32, [vp, vp, i64, i32, i32, vp, vp, i64, i32, vp, vp]),
        "psd_kernel_attention_scratch_bytes": (i64, [i32, i32, i32, i32]),
        "psd_kernel_attention_bf16": (i32, [vp, i32, i32, i32, i32, i32, i32, vp, vp, vp]),
        "psd_kernel_head_scratch_bytes": (i64, [i32, i32]),
        "psd_kernel_head_confidence_bf16": (i32, [vp, vp, i32, i32, i32, C.c_float, i32, vp, vp, vp, vp]),
        "psd_debug_force_gemm_tile": (i32, [i32]),
        "psd_debug_set_graphs": (i32, [vp, i32, C.POINTER(i64)]),
        "psd_kernel_packed_bytes": (i64, [i64, i32]),
        "psd_kernel_pack_rows": (i32, [vp, i64, i32, vp, vp]),
        "psd_kernel_head_stream_bf16": (i32, [vp, vp, i32, i32, i32, C.c_float, i32, vp, vp, vp, vp]),
        "psd_kernel_head_stream_static_bf16": (i32, [vp, vp, i32, i32, i32, C.c_float, i32, vp, vp, vp]),
        "psd_kernel_mfma_rate": (i32, [vp, i64, i32, vp, i64, C.POINTER(C.c_double), vp]),
        "psd_probe_begin": (i32, [vp, i32, i32, i32]),
        "psd_probe_end": (i32, [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double)]),
        "psd_probe_read": (i32, [vp, i32, i32, C.POINTER(C.c_float), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]),
        "psd_kernel_gemm_tile": (i32, [i64, i32, i32]),
        "psd_kernel_gemm_tile_count": (i32, []),
        "psd_kernel_gemm_tile_name": (C.c_char_p, [i32]),
        "psd_forward_work": (i32, [C.POINTER(_Config), i32, i32, i32, C.POINTER(_Work)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    # the structures declared here must be the ones the library was built with
    mine = [C.sizeof(t) for t in (_Config, _Weights, _Policy, _Graph, _Stats, _Work, _GraphScore, _DebugLayout)]
    theirs = (i32 * len(mine))()
    if lib.psd_struct_sizes(theirs, len(mine)) != len(mine) or list(theirs) != mine:
        raise PsdError(f"binding and libpsd.so disagree on the structure layouts: {mine} vs {list(theirs)} (rebuild the library)")
    _lib = lib
    return lib


def _check(rc: int):
    if rc < 0:
        lib = load_library()
        raise PsdError(f"{lib.psd_status_string(int(rc)).decode()} ({int(rc)}): {lib.psd_last_error().decode()}")
    return rc


@dataclass(frozen=True)
class Policy:
    tau: float = 0.9
    k_min: int = 1
    k_max: int = 0
    eos_id: Optional[int] = None     # EOS early stopping of the block loop (App. B.1); None = off
    # block loops: the post-verification commit doubles as the next stage-1 commit and the next drafts come from the
    # accepted draft's verifier output -- one model call per iteration; not the literal Alg. 1
    single_forward: bool = False

    def c(self) -> _Policy:
        return _Policy(float(np.float32(self.tau)), int(self.k_min), int(self.k_max),
                       0 if self.eos_id is None else 1, 0 if self.eos_id is None else int(self.eos_id),
                       1 if self.single_forward else 0)


@dataclass(frozen=True)
class Graph:
    rank_sets: tuple      # K ints, bit r set <-> rank r speculated; rank_sets[0] == 0

    @property
    def K(self) -> int:
        return len(self.rank_sets)

    def c(self) -> _Graph:
        g = _Graph()
        g.K = self.K
        for k, bits in enumerate(self.rank_sets):
            g.rank_set[k] = int(bits)
        return g


def chain_graph(K: int, width: int = 1) -> Graph:
    g = _Graph()
    _check(load_library().psd_graph_chain(K, width, C.byref(g)))
    return Graph(tuple(int(g.rank_set[k]) for k in range(g.K)))


def lattice_graph(depth: int) -> Graph:
    g = _Graph()
    _check(load_library().psd_graph_lattice(depth, C.byref(g)))
    return Graph(tuple(int(g.rank_set[k]) for k in range(g.K)))


@dataclass
class Stats:
    invocations: int = 0
    tokens_policy: int = 0
    tokens_draft: int = 0
    tokens_postverify: int = 0
    depth_hist: List[int] = field(default_factory=lambda: [0] * HIST)
    tokens_counted: int = 0      # resolved positions at or before the EOS position (App. B.1)
    stopped: bool = False
    eos_pos: int = -1

    @property
    def tokens(self) -> int:
        return self.tokens_policy + self.tokens_draft + self.tokens_postverify

    @property
    def tpf(self) -> float:
        return self.tokens / max(1, self.invocations)

    @property
    def tpf_counted(self) -> float:
        return self.tokens_counted / max(1, self.invocations)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_i32(t, device):
    return torch.as_tensor(np.ascontiguousarray(t, dtype=np.int32) if not torch.is_tensor(t) else t, device=device) \
        .to(torch.int32).contiguous()


def pack_qkv(lt: dict) -> None:
    """Re-homes wq | wk | wv (and bq | bk | bv) of one layer back to back in one allocation, so the
    library can run the three projections as a single contraction, and w_down into padded rows.
    Views keep the storage alive."""
    w = torch.cat([lt["wq"], lt["wk"], lt["wv"]], dim=0).contiguous()
    nq, nk = lt["wq"].shape[0], lt["wk"].shape[0]
    lt["wq"], lt["wk"], lt["wv"] = w[:nq], w[nq:nq + nk], w[nq + nk:]
    if lt.get("bq") is not None:
        b = torch.cat([lt["bq"], lt["bk"], lt["bv"]]).contiguous()
        lt["bq"], lt["bk"], lt["bv"] = b[:nq], b[nq:nq + nk], b[nq + nk:]
    # w_down [d_model, d_ffn] with rows padded by 64 elements: dense rows of a multiple of 8 KB would all start
    # in the same cache channel (see psd_weights.w_down_stride)
    wd = lt["w_down"]
    if wd.dtype == torch.bfloat16 and wd.stride(0) == wd.shape[1]:
        padded = torch.zeros((wd.shape[0], wd.shape[1] + 64), dtype=wd.dtype, device=wd.device)
        padded[:, :wd.shape[1]] = wd
        lt["w_down"] = padded[:, :wd.shape[1]]


class Model:
    """Device-resident weights plus the library handle.  ``Model.from_host(host_model)``
    uploads a psd_inputs.HostModel; matrices go up in the model dtype, the rest as fp32."""

    def __init__(self, shape, max_seq: int, tensors: dict, layer_tensors: list, device="cuda:0"):
        self.lib = load_library()
        self.shape = shape
        self.max_seq = int(max_seq)
        self.device = torch.device(device)
        self._tensors = tensors            # keep alive: the handle borrows the pointers
        self._layers = layer_tensors
        self._ws = None
        cfg = _Config(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.d_head, shape.d_ffn,
                      shape.vocab, shape.mask_id, shape.rms_eps, int(shape.qkv_bias), 1 if shape.dtype == "bf16" else 0,
                      float(shape.logit_scale), self.max_seq, 1 if getattr(shape, "attention", "bidirectional") == "block_causal" else 0)
        self.cfg = cfg
        self._check_tensors(shape, mat_dtype=torch.bfloat16 if shape.dtype == "bf16" else torch.float32)
        w = _Weights()
        for name in ("tok_emb", "final_norm", "lm_head", "rope_cos", "rope_sin"):
            setattr(w, name, tensors[name].data_ptr())
        self._arrays = {}
        for name in ("attn_norm", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
            if layer_tensors[0].get(name) is None:
                setattr(w, name, None)
                continue
            arr = (C.c_void_p * shape.n_layers)(*[lt[name].data_ptr() for lt in layer_tensors])
            self._arrays[name] = arr
            setattr(w, name, C.cast(arr, _PP))
        strides = {lt["w_down"].stride(0) for lt in layer_tensors}
        assert len(strides) == 1 and all(lt["w_down"].stride(1) == 1 for lt in layer_tensors)
        w.w_down_stride = strides.pop()
        handle = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(self.lib.psd_create(C.byref(cfg), C.byref(w), C.byref(handle)))
        self.handle = handle

    def _check_tensors(self, shape, mat_dtype):
        """The library takes raw pointers: a tensor of the wrong dtype or extent would be read as garbage or past its
        end.  Matrices [out, in] in the model dtype; norm gains, biases and rotary tables fp32."""
        d, hq, hkv, f, v = shape.d_model, shape.n_heads * shape.d_head, shape.n_kv_heads * shape.d_head, shape.d_ffn, shape.vocab
        want = {"tok_emb": ((v, d), mat_dtype), "lm_head": ((v, d), mat_dtype), "final_norm": ((d,), torch.float32),
                "rope_cos": ((self.max_seq, shape.d_head // 2), torch.float32),
                "rope_sin": ((self.max_seq, shape.d_head // 2), torch.float32)}
        per_layer = {"attn_norm": ((d,), torch.float32), "ffn_norm": ((d,), torch.float32), "wq": ((hq, d), mat_dtype),
                     "wk": ((hkv, d), mat_dtype), "wv": ((hkv, d), mat_dtype), "wo": ((d, hq), mat_dtype),
                     "w_gate": ((f, d), mat_dtype), "w_up": ((f, d), mat_dtype), "w_down": ((d, f), mat_dtype),
                     "bq": ((hq,), torch.float32), "bk": ((hkv,), torch.float32), "bv": ((hkv,), torch.float32)}

        def check(name, t, dims, dtype, dense=True):
            if tuple(t.shape) != tuple(dims) or t.dtype != dtype or t.device.type != self.device.type or t.stride(-1) != 1 \
                    or (dense and not t.is_contiguous()):
                raise PsdError(f"{name}: expected a {'dense ' if dense else ''}{dtype} tensor of shape {tuple(dims)} on {self.device}, "
                               f"got {t.dtype} {tuple(t.shape)} strides {t.stride()} on {t.device}")
        for name, (dims, dtype) in want.items():
            check(name, self._tensors[name], dims, dtype)
        for l, lt in enumerate(self._layers):
            for name, (dims, dtype) in per_layer.items():
                if lt.get(name) is None:
                    if name in ("bq", "bk", "bv") and not shape.qkv_bias:
                        continue
                    raise PsdError(f"layer {l}: {name} is missing")
                check(f"layer {l} {name}", lt[name], dims, dtype, dense=(name != "w_down"))

    @classmethod
    def from_host(cls, host_model, device="cuda:0") -> "Model":
        shape = host_model.shape
        mat_dtype = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        dev = torch.device(device)

        def up(a, dtype):
            return torch.from_numpy(np.ascontiguousarray(a)).to(device=dev, dtype=dtype).contiguous()

        tensors = {"tok_emb": up(host_model.tok_emb, mat_dtype), "lm_head": up(host_model.lm_head, mat_dtype),
                   "final_norm": up(host_model.final_norm, torch.float32),
                   "rope_cos": up(host_model.rope_cos, torch.float32), "rope_sin": up(host_model.rope_sin, torch.float32)}
        layers = []
        for lw in host_model.layers:
            lt = {}
            for k, v in lw.items():
                if v is None:
                    lt[k] = None
                else:
                    lt[k] = up(v, mat_dtype if v.ndim == 2 else torch.float32)
            pack_qkv(lt)
            layers.append(lt)
        return cls(shape, host_model.max_seq, tensors, layers, device)

    def close(self):
        if getattr(self, "handle", None):
            self.lib.psd_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_plain(self, mask: int):
        _check(self.lib.psd_debug_set_plain(self.handle, int(mask)))

    def set_graphs(self, enabled: Optional[bool] = None) -> int:
        """Switches the HIP-graph replay of the block loops' model calls on / off (None: leave); returns the number of
        graph launches so far."""
        n = C.c_int64()
        _check(self.lib.psd_debug_set_graphs(self.handle, -1 if enabled is None else int(bool(enabled)), C.byref(n)))
        return int(n.value)

    def probe_begin(self, epilogue: int, tile: int, max_launches: int = 65536):
        _check(self.lib.psd_probe_begin(self.handle, epilogue, tile, max_launches))

    def probe_end(self, epilogue: int):
        ms, n, fl = C.c_double(), C.c_int64(), C.c_double()
        _check(self.lib.psd_probe_end(self.handle, epilogue, C.byref(ms), C.byref(n), C.byref(fl)))
        return ms.value, n.value, fl.value

    def probe_read(self, epilogue: int, max_n: int = 1 << 16):
        """Per timed launch of the last probe of this kind: (milliseconds, a, b) -- see psd_probe_read."""
        ms, a, b = (C.c_float * max_n)(), (C.c_int64 * max_n)(), (C.c_int64 * max_n)()
        n = self.lib.psd_probe_read(self.handle, epilogue, max_n, ms, a, b)
        _check(n)
        return [(float(ms[i]), int(a[i]), int(b[i])) for i in range(n)]

    def workspace(self, n_bytes: int) -> torch.Tensor:
        if self._ws is None or self._ws.numel() < n_bytes:
            self._ws = None
            self._ws = torch.empty(int(n_bytes) + 256, dtype=torch.uint8, device=self.device)
        return self._ws

    def forward_ws(self, S: int, N: int, L: int, extra: int = 0):
        need = self.lib.psd_workspace_bytes(C.byref(self.cfg), S, N, L)
        _check(need)
        ws = self.workspace(need + extra)
        return ws, need + extra


def forward_work(model: Model, S: int, N: int, L: int) -> dict:
    w = _Work()
    _check(model.lib.psd_forward_work(C.byref(model.cfg), S, N, L, C.byref(w)))
    return {k: getattr(w, k) for k, _ in _Work._fields_}


# ------------------------------------------------------------------------------------------
# the calls of include/psd.h
# ------------------------------------------------------------------------------------------


def psd_forward_confidence(model: Model, tokens: torch.Tensor, block_start: int, L: int):
    """tokens int32 [S, N] on the device -> (top1 int32 [S, L], conf float32 [S, L])."""
    assert tokens.dtype == torch.int32 and tokens.is_contiguous() and tokens.dim() == 2
    S, N = tokens.shape
    top1 = torch.empty((S, L), dtype=torch.int32, device=tokens.device)
    conf = torch.empty((S, L), dtype=torch.float32, device=tokens.device)
    ws, nb = model.forward_ws(S, N, L)
    _check(model.lib.psd_forward_confidence(model.handle, _ptr(tokens), S, N, block_start, L, _ptr(top1), _ptr(conf),
                                            _ptr(ws), nb, _stream()))
    return top1, conf


def psd_forward_logits(model: Model, tokens: torch.Tensor, block_start: int, L: int) -> torch.Tensor:
    assert tokens.dtype == torch.int32 and tokens.is_contiguous() and tokens.dim() == 2
    S, N = tokens.shape
    logits = torch.empty((S * L, model.shape.vocab), dtype=torch.float32, device=tokens.device)
    ws, nb = model.forward_ws(S, N, L)
    _check(model.lib.psd_forward_logits(model.handle, _ptr(tokens), S, N, block_start, L, _ptr(logits), _ptr(ws), nb,
                                        _stream()))
    return logits


def psd_select_unmask(model: Model, tokens: torch.Tensor, block_start: int, L: int, top1: torch.Tensor,
                      conf: torch.Tensor, policy: Policy):
    """In place on tokens [B, N]; returns (transfer_mask uint8 [B, L], n_selected int32 [B])."""
    B, N = tokens.shape
    tm = torch.empty((B, L), dtype=torch.uint8, device=tokens.device)
    ns = torch.empty((B,), dtype=torch.int32, device=tokens.device)
    pol = policy.c()
    _check(model.lib.psd_select_unmask(model.handle, _ptr(tokens), B, N, block_start, L, _ptr(top1), _ptr(conf),
                                       C.byref(pol), _ptr(tm), _ptr(ns), _stream()))
    return tm, ns


def psd_build_drafts(model: Model, tokens: torch.Tensor, block_start: int, L: int, top1: torch.Tensor,
                     conf: torch.Tensor, graph: Graph):
    """-> (sigma int32 [B, L], m int32 [B], drafts int32 [B, K, N])."""
    B, N = tokens.shape
    sigma = torch.empty((B, L), dtype=torch.int32, device=tokens.device)
    m = torch.empty((B,), dtype=torch.int32, device=tokens.device)
    drafts = torch.empty((B, graph.K, N), dtype=torch.int32, device=tokens.device)
    g = graph.c()
    _check(model.lib.psd_build_drafts(model.handle, _ptr(tokens), B, N, block_start, L, _ptr(top1), _ptr(conf),
                                      C.byref(g), _ptr(sigma), _ptr(m), _ptr(drafts), _stream()))
    return sigma, m, drafts


def psd_accept(model: Model, tokens: torch.Tensor, drafts: torch.Tensor, block_start: int, L: int, sigma: torch.Tensor,
               m: torch.Tensor, graph: Graph, policy: Policy, v_top1: torch.Tensor, v_conf: torch.Tensor):
    """In place on tokens; returns (k_star int32 [B], accepted uint8 [B, K])."""
    B, N = tokens.shape
    k_star = torch.empty((B,), dtype=torch.int32, device=tokens.device)
    accepted = torch.empty((B, graph.K), dtype=torch.uint8, device=tokens.device)
    g, pol = graph.c(), policy.c()
    _check(model.lib.psd_accept(model.handle, _ptr(tokens), _ptr(drafts), B, N, block_start, L, _ptr(sigma), _ptr(m),
                                C.byref(g), C.byref(pol), _ptr(v_top1), _ptr(v_conf), _ptr(k_star), _ptr(accepted),
                                _stream()))
    return k_star, accepted


def psd_verify_accept(model: Model, tokens: torch.Tensor, drafts: torch.Tensor, block_start: int, L: int,
                      sigma: torch.Tensor, m: torch.Tensor, graph: Graph, policy: Policy):
    """One batched forward over the drafts + acceptance; in place on tokens.
    Returns (k_star, accepted, v_top1 [B, K, L], v_conf [B, K, L])."""
    B, N = tokens.shape
    K = graph.K
    k_star = torch.empty((B,), dtype=torch.int32, device=tokens.device)
    accepted = torch.empty((B, K), dtype=torch.uint8, device=tokens.device)
    v_top1 = torch.empty((B, K, L), dtype=torch.int32, device=tokens.device)
    v_conf = torch.empty((B, K, L), dtype=torch.float32, device=tokens.device)
    g, pol = graph.c(), policy.c()
    ws, nb = model.forward_ws(B * K, N, L)
    _check(model.lib.psd_verify_accept(model.handle, _ptr(tokens), _ptr(drafts), B, N, block_start, L, _ptr(sigma),
                                       _ptr(m), C.byref(g), C.byref(pol), _ptr(k_star), _ptr(accepted), _ptr(v_top1),
                                       _ptr(v_conf), _ptr(ws), nb, _stream()))
    return k_star, accepted, v_top1, v_conf


def _add_stats(stats, cstats, B) -> List[Stats]:
    out = list(stats) if stats is not None else [Stats() for _ in range(B)]
    for b in range(B):
        out[b].invocations += cstats[b].invocations
        out[b].tokens_policy += cstats[b].tokens_policy
        out[b].tokens_draft += cstats[b].tokens_draft
        out[b].tokens_postverify += cstats[b].tokens_postverify
        out[b].tokens_counted += cstats[b].tokens_counted
        if cstats[b].stopped:
            out[b].stopped, out[b].eos_pos = True, int(cstats[b].eos_pos)
        for i in range(HIST):
            out[b].depth_hist[i] += cstats[b].depth_hist[i]
    return out


def _starts(block_start, B: int):
    """One block start for the whole batch, or one per sequence -> int32[B] for the C call."""
    vals = [int(block_start)] * B if np.isscalar(block_start) else [int(v) for v in block_start]
    if len(vals) != B:
        raise PsdError(f"{len(vals)} block starts for a batch of {B}")
    return (C.c_int32 * B)(*vals)


def psd_decode_block(model: Model, tokens: torch.Tensor, block_start, L: int, policy: Policy, graph: Graph,
                     stats: Optional[Sequence[Stats]] = None) -> List[Stats]:
    """Alg. 1 on one block of every sequence of tokens [B, N], in place; block_start is one position for the batch or one
    per sequence.  Blocks until done."""
    B, N = tokens.shape
    K = graph.K
    extra = model.lib.psd_decode_scratch_bytes(B, N, L, K)
    _check(extra)
    ws, nb = model.forward_ws(B * K, N, L, extra=extra)
    cstats = (_Stats * B)()
    g, pol = graph.c(), policy.c()
    _check(model.lib.psd_decode_block(model.handle, _ptr(tokens), B, N, _starts(block_start, B), L, C.byref(pol), C.byref(g),
                                      cstats, _ptr(ws), nb, _stream()))
    return _add_stats(stats, cstats, B)


def psd_decode(model: Model, tokens: torch.Tensor, block_start, L: int, policy: Policy, graph: Graph,
               stats: Optional[Sequence[Stats]] = None, max_iterations: int = 0):
    """The whole generation behind one call: every sequence walks through its own blocks (see psd.h).  block_start as for
    psd_decode_block.  Returns (stats, block starts on return, iterations run); with max_iterations > 0 the call returns
    after that many iterations and can be continued from the returned block starts."""
    B, N = tokens.shape
    K = graph.K
    extra = model.lib.psd_decode_scratch_bytes(B, N, L, K)
    _check(extra)
    ws, nb = model.forward_ws(B * K, N, L, extra=extra)
    cstats = (_Stats * B)()
    g, pol = graph.c(), policy.c()
    starts = _starts(block_start, B)
    done = C.c_int32(0)
    _check(model.lib.psd_decode(model.handle, _ptr(tokens), B, N, starts, L, C.byref(pol), C.byref(g), cstats,
                                int(max_iterations), C.byref(done), _ptr(ws), nb, _stream()))
    return _add_stats(stats, cstats, B), [int(v) for v in starts], int(done.value)


class KvCache:
    """Device memory for the prefix KV caches of n_seqs sequences of a context-causal block model (zeroed)."""

    def __init__(self, model: Model, n_seqs: int, capacity: int):
        per_seq = model.lib.psd_kv_cache_bytes(C.byref(model.cfg), capacity)
        _check(per_seq)
        self.model, self.n_seqs, self.capacity = model, n_seqs, capacity
        self.mem = torch.empty(per_seq * n_seqs + 256, dtype=torch.uint8, device=model.device)
        self.reset()

    def reset(self):
        _check(self.model.lib.psd_kv_reset(self.model.handle, _ptr(self.mem), self.n_seqs, self.capacity, _stream()))


def psd_kv_prefill(model: Model, tokens: torch.Tensor, n_prompt: int, L: int, cache: KvCache) -> None:
    B, N = tokens.shape
    ws, nb = model.forward_ws(B, L, L)
    _check(model.lib.psd_kv_prefill(model.handle, _ptr(tokens), B, N, n_prompt, L, _ptr(cache.mem), cache.capacity, _ptr(ws), nb,
                                    _stream()))


def psd_forward_confidence_cached(model: Model, tokens: torch.Tensor, block_start: int, L: int, cache: KvCache,
                                  seqs_per_cache: int = 1, want_logits: bool = False):
    """tokens int32 [S, N]; the block rows against the caches -> (top1 [S, L], conf [S, L][, logits [S*L, V]])."""
    S, N = tokens.shape
    top1 = torch.empty((S, L), dtype=torch.int32, device=tokens.device)
    conf = torch.empty((S, L), dtype=torch.float32, device=tokens.device)
    logits = torch.empty((S * L, model.shape.vocab), dtype=torch.float32, device=tokens.device) if want_logits else None
    ws, nb = model.forward_ws(S, L, L)
    _check(model.lib.psd_forward_confidence_cached(model.handle, _ptr(tokens), S, N, block_start, L, seqs_per_cache,
                                                   _ptr(cache.mem), cache.capacity, _ptr(top1), _ptr(conf), _ptr(logits),
                                                   _ptr(ws), nb, _stream()))
    return (top1, conf, logits) if want_logits else (top1, conf)


def psd_decode_block_cached(model: Model, tokens: torch.Tensor, block_start: int, L: int, policy: Policy, graph: Graph,
                            cache: KvCache, stats: Optional[Sequence[Stats]] = None) -> List[Stats]:
    """psd_decode_block with cached model calls; the finished block is appended to the caches."""
    B, N = tokens.shape
    K = graph.K
    extra = model.lib.psd_decode_scratch_bytes(B, N, L, K)
    _check(extra)
    ws, nb = model.forward_ws(B * K, L, L, extra=extra)
    cstats = (_Stats * B)()
    g, pol = graph.c(), policy.c()
    _check(model.lib.psd_decode_block_cached(model.handle, _ptr(tokens), B, N, block_start, L, C.byref(pol), C.byref(g), cstats,
                                             _ptr(cache.mem), cache.capacity, _ptr(ws), nb, _stream()))
    return _add_stats(stats, cstats, B)


def psd_forward_confidence_approx(model: Model, tokens: torch.Tensor, block_start: int, L: int, cache: KvCache, refresh: bool,
                                  seqs_per_cache: int = 1, want_logits: bool = False):
    """Model call of a bidirectional model under the approximate prefix + suffix cache: refresh = exact call over the whole
    sequences that fills the caches; otherwise the block rows against them.  Returns (top1, conf[, logits])."""
    S, N = tokens.shape
    ws, nb = model.forward_ws(S, N if refresh else L, L)
    top1 = torch.empty((S, L), dtype=torch.int32, device=tokens.device)
    conf = torch.empty((S, L), dtype=torch.float32, device=tokens.device)
    logits = torch.empty((S * L, model.cfg.vocab), dtype=torch.float32, device=tokens.device) if want_logits else None
    _check(model.lib.psd_forward_confidence_approx(model.handle, _ptr(tokens), S, N, block_start, L, 1 if refresh else 0,
                                                   seqs_per_cache, _ptr(cache.mem), cache.capacity, _ptr(top1), _ptr(conf),
                                                   _ptr(logits), _ptr(ws), nb, _stream()))
    return (top1, conf, logits) if want_logits else (top1, conf)


def psd_decode_block_approx(model: Model, tokens: torch.Tensor, block_start: int, L: int, policy: Policy, graph: Graph,
                            cache: KvCache, stats: Optional[Sequence[Stats]] = None) -> List[Stats]:
    """psd_decode_block under the approximate cache: the first model call on the block is exact and fills the caches."""
    B, N = tokens.shape
    K = graph.K
    extra = model.lib.psd_decode_scratch_bytes(B, N, L, K)
    _check(extra)
    full = model.lib.psd_workspace_bytes(C.byref(model.cfg), B, N, L)
    rows = model.lib.psd_workspace_bytes(C.byref(model.cfg), B * K, L, L)
    _check(full)
    _check(rows)
    if full >= rows:
        ws, nb = model.forward_ws(B, N, L, extra=extra)
    else:
        ws, nb = model.forward_ws(B * K, L, L, extra=extra)
    cstats = (_Stats * B)()
    g, pol = graph.c(), policy.c()
    _check(model.lib.psd_decode_block_approx(model.handle, _ptr(tokens), B, N, block_start, L, C.byref(pol), C.byref(g), cstats,
                                             _ptr(cache.mem), cache.capacity, _ptr(ws), nb, _stream()))
    return _add_stats(stats, cstats, B)


def psd_calibrate_graph(model: Model, tokens: torch.Tensor, prompt_len: int, L: int, policy: Policy,
                        candidates: Sequence[Graph], cache: Optional[KvCache] = None):
    """Offline choice of the draft graph: decodes the calibration batch tokens [B, N] (left untouched) once per
    candidate and returns (index of the candidate with the highest tokens/s, list of score dicts)."""
    B, N = tokens.shape
    K = max(g.K for g in candidates)
    extra = model.lib.psd_decode_scratch_bytes(B, N, L, K)
    _check(extra)
    ws, nb = model.forward_ws(B * K, N, L, extra=extra)
    work = torch.empty_like(tokens)
    cg = (_Graph * len(candidates))(*[g.c() for g in candidates])
    scores = (_GraphScore * len(candidates))()
    best = C.c_int32(-1)
    pol = policy.c()
    _check(model.lib.psd_calibrate_graph(model.handle, _ptr(tokens), _ptr(work), B, N, prompt_len, L, C.byref(pol), cg,
                                         len(candidates), scores, C.byref(best), None if cache is None else _ptr(cache.mem),
                                         0 if cache is None else cache.capacity, _ptr(ws), nb, _stream()))
    return int(best.value), [{k: getattr(sc, k) for k, _ in _GraphScore._fields_} for sc in scores]


def decode(model: Model, tokens: torch.Tensor, prompt_len: int, L: int, policy: Policy, graph: Graph) -> List[Stats]:
    """Semi-autoregressive generation of everything behind the prompt: one psd_decode call (every sequence walks through
    its own blocks; with EOS early stopping a sequence ends with the block that produced the EOS token).  A generated
    part that is not whole blocks is decoded block by block with a shorter last block."""
    B, N = tokens.shape
    if (N - prompt_len) % L == 0:
        return psd_decode(model, tokens, prompt_len, L, policy, graph)[0]
    stats = [Stats() for _ in range(B)]
    for block_start in range(prompt_len, N, L):
        if all(s.stopped for s in stats):
            break
        if any(s.stopped for s in stats):
            raise PsdError("a ragged last block after an EOS stop of part of the batch: decode those sequences separately")
        stats = psd_decode_block(model, tokens, block_start, min(L, N - block_start), policy, graph, stats)
    return stats


# ------------------------------------------------------------------------------------------
# kernel-level hooks (parity tests and timing at full shapes without a model)
# ------------------------------------------------------------------------------------------

EPI_STORE, EPI_BIAS, EPI_RESIDUAL, EPI_SWIGLU = 0, 1, 2, 3


def debug_layer(model: Model, layer: int, hidden: torch.Tensor, S: int, N: int, L: int, stop_after: int = 0) -> dict:
    """psd_debug_layer: one layer of the model on the caller's residual stream hidden fp32 [S*N, d_model] (in place).
    Returns views of the intermediates the layer left in the workspace (valid until the next call on this model):
    a [S*N, d], qkv [S*N, qkv_w] (rotary applied), o [S*N, H*dh], act [S*N, d_ffn] (stop_after = 0 only)."""
    assert hidden.dtype == torch.float32 and hidden.is_contiguous() and hidden.shape == (S * N, model.shape.d_model)
    ws, nb = model.forward_ws(S, N, L)
    lay = _DebugLayout()
    _check(model.lib.psd_debug_workspace_layout(C.byref(model.cfg), S, N, L, C.byref(lay)))
    _check(model.lib.psd_debug_layer(model.handle, layer, _ptr(hidden), S, N, L, stop_after, _ptr(ws), nb, _stream()))
    sh = model.shape
    dt = torch.bfloat16 if sh.dtype == "bf16" else torch.float32
    esz = 2 if sh.dtype == "bf16" else 4
    T = S * N
    qkv_w = (sh.n_heads + 2 * sh.n_kv_heads) * sh.d_head

    def view(off, rows, ld, width):
        return ws[off: off + rows * ld * esz].view(dt).view(rows, ld)[:, :width]

    out = {"a": view(lay.off_a, T, sh.d_model, sh.d_model), "qkv": view(lay.off_qkv, T, lay.ld_qkv, qkv_w),
           "o": view(lay.off_o, T, sh.n_heads * sh.d_head, sh.n_heads * sh.d_head)}
    if stop_after == 0:
        out["act"] = view(lay.off_act, T, lay.ld_act, sh.d_ffn)
    return out


# ------------------------------------------------------------------------------------------
# kernel-level hooks (parity tests and timing at full shapes without a model)
# ------------------------------------------------------------------------------------------

EPI_STORE, EPI_BIAS, EPI_RESIDUAL, EPI_SWIGLU = 0, 1, 2, 3


def kernel_gemm_bf16(A: torch.Tensor, W: torch.Tensor, epilogue: int = EPI_STORE, W2: Optional[torch.Tensor] = None,
                     bias: Optional[torch.Tensor] = None, resid: Optional[torch.Tensor] = None,
                     out: Optional[torch.Tensor] = None):
    """A bf16 [M, K], W bf16 [N, K] -> out bf16 [M, N] (or resid fp32 [M, N] += for EPI_RESIDUAL).
    A and W (W2 like W) may be row-strided views (unit stride along K)."""
    lib = load_library()
    M, K = A.shape
    Nout = W.shape[0]
    assert A.stride(1) == 1 and W.stride(1) == 1 and (W2 is None or W2.stride() == W.stride())
    lda, ldw = A.stride(0), W.stride(0)
    if epilogue == EPI_RESIDUAL:
        assert resid is not None and resid.dtype == torch.float32
        _check(lib.psd_kernel_gemm_bf16(_ptr(A), _ptr(W), None, M, Nout, K, lda, ldw, epilogue, None, None, _ptr(resid),
                                        resid.stride(0), _stream()))
        return resid
    if out is None:
        out = torch.empty((M, Nout), dtype=torch.bfloat16, device=A.device)
    _check(lib.psd_kernel_gemm_bf16(_ptr(A), _ptr(W), _ptr(W2), M, Nout, K, lda, ldw, epilogue, _ptr(bias), _ptr(out), None,
                                    out.stride(0), _stream()))
    return out


def kernel_gemm_residual_splitk(A: torch.Tensor, W: torch.Tensor, resid: torch.Tensor, k_splits: int = 0,
                                partial: Optional[torch.Tensor] = None) -> int:
    """resid fp32 [M, N] += A W^T with the K range cut into k_splits parts (0 = the forward's choice);
    returns the number of parts used."""
    lib = load_library()
    M, K = A.shape
    Nout = W.shape[0]
    assert A.is_contiguous() and W.is_contiguous()
    assert resid.dtype == torch.float32 and resid.is_contiguous() and resid.shape == (M, Nout)
    if partial is None:
        partial = torch.empty((7 * M * Nout,), dtype=torch.float32, device=A.device)
    used = C.c_int32(0)
    _check(lib.psd_kernel_gemm_residual_splitk(_ptr(A), _ptr(W), M, Nout, K, _ptr(resid), _ptr(partial),
                                               partial.numel() * 4, k_splits, C.byref(used), _stream()))
    return used.value


def kernel_attention_bf16(qkv: torch.Tensor, S: int, N: int, n_heads: int, n_kv_heads: int, d_head: int,
                          out: Optional[torch.Tensor] = None, vT: Optional[torch.Tensor] = None):
    """qkv bf16 [S*N, (n_heads + 2 n_kv_heads) * d_head], possibly a row-strided view -> out bf16 [S*N, n_heads*d_head]."""
    lib = load_library()
    assert qkv.stride(1) == 1
    if vT is None:
        vT = torch.empty((lib.psd_kernel_attention_scratch_bytes(S, N, n_kv_heads, d_head) // 2,), dtype=torch.bfloat16,
                         device=qkv.device)
    if out is None:
        out = torch.empty((S * N, n_heads * d_head), dtype=torch.bfloat16, device=qkv.device)
    _check(lib.psd_kernel_attention_bf16(_ptr(qkv), qkv.stride(0), S, N, n_heads, n_kv_heads, d_head, _ptr(vT), _ptr(out),
                                         _stream()))
    return out


def kernel_head_confidence_bf16(y: torch.Tensor, W: torch.Tensor, scale: float, mask_id: int, scratch=None):
    """y bf16 [rows, d], W bf16 [V, d] -> (row_sum fp32 [rows], row_arg int32 [rows])."""
    lib = load_library()
    rows, d = y.shape
    V = W.shape[0]
    if scratch is None:
        scratch = torch.empty((int(lib.psd_kernel_head_scratch_bytes(rows, V)),), dtype=torch.uint8, device=y.device)
    row_sum = torch.empty((rows,), dtype=torch.float32, device=y.device)
    row_arg = torch.empty((rows,), dtype=torch.int32, device=y.device)
    _check(lib.psd_kernel_head_confidence_bf16(_ptr(y), _ptr(W), rows, V, d, float(scale), int(mask_id), _ptr(scratch),
                                               _ptr(row_sum), _ptr(row_arg), _stream()))
    return row_sum, row_arg


def kernel_mfma_rate(operands: torch.Tensor, iters: int = 4000) -> float:
    """Sustained TFLOP/s of a pure-MFMA loop on the given bf16 operand data (see psd.h)."""
    lib = load_library()
    sink = torch.empty((4 << 20,), dtype=torch.uint8, device=operands.device)
    fl = C.c_double()
    nbytes = operands.numel() * operands.element_size()
    _check(lib.psd_kernel_mfma_rate(_ptr(operands), nbytes, 50, _ptr(sink), sink.numel(), C.byref(fl), _stream()))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    _check(lib.psd_kernel_mfma_rate(_ptr(operands), nbytes, iters, _ptr(sink), sink.numel(), C.byref(fl), _stream()))
    e1.record()
    torch.cuda.synchronize()
    return fl.value / (e0.elapsed_time(e1) * 1e-3) / 1e12


def kernel_pack_rows(src: torch.Tensor) -> torch.Tensor:
    """Row-major bf16 [R, K] -> its MFMA-fragment-order copy (flat bf16 tensor)."""
    lib = load_library()
    R, K = src.shape
    n = int(lib.psd_kernel_packed_bytes(R, K))
    _check(n)
    dst = torch.empty((n // 2,), dtype=torch.bfloat16, device=src.device)
    _check(lib.psd_kernel_pack_rows(_ptr(src), R, K, _ptr(dst), _stream()))
    return dst


def kernel_head_stream_bf16(y: torch.Tensor, W_packed: torch.Tensor, V: int, scale: float, mask_id: int, scratch=None,
                            y_packed=None):
    """Streaming LM-head on a pre-packed weight copy; y row-major bf16 [rows, d] is packed here."""
    lib = load_library()
    rows, d = y.shape
    if y_packed is None:
        y_packed = kernel_pack_rows(y)
    if scratch is None:
        scratch = torch.empty((int(lib.psd_kernel_head_scratch_bytes(rows, V)),), dtype=torch.uint8, device=y.device)
    row_sum = torch.empty((rows,), dtype=torch.float32, device=y.device)
    row_arg = torch.empty((rows,), dtype=torch.int32, device=y.device)
    _check(lib.psd_kernel_head_stream_bf16(_ptr(y_packed), _ptr(W_packed), rows, V, d, float(scale), int(mask_id),
                                           _ptr(scratch), _ptr(row_sum), _ptr(row_arg), _stream()))
    return row_sum, row_arg


def kernel_head_stream_static_bf16(y_packed: torch.Tensor, W_packed: torch.Tensor, rows: int, V: int, d: int, scale: float,
                                   mask_id: int, row_sum: torch.Tensor, row_arg: torch.Tensor) -> None:
    """psd_kernel_head_stream_static_bf16: every buffer comes from the caller, the library's static array serves as
    scratch; nothing is allocated here or in the library."""
    _check(load_library().psd_kernel_head_stream_static_bf16(_ptr(y_packed), _ptr(W_packed), rows, V, d, float(scale),
                                                             int(mask_id), _ptr(row_sum), _ptr(row_arg), _stream()))
