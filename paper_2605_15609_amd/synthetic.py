"""Device models with seeded synthetic weights (drawn by psd_inputs), uploaded tensor by
tensor so that an 8B-parameter model never needs its fp32 host copy in one piece."""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

import psd_inputs as inp
from .binding import Model, pack_qkv


def synthetic_model(shape: "inp.ModelShape", max_seq: int, device: str = "cuda:0", threads: int = 8) -> Model:
    dev = torch.device(device)
    mat_dtype = torch.bfloat16 if shape.dtype == "bf16" else torch.float32

    def up(a, matrix=None):
        # weight matrices go up in the model dtype; norm gains, biases and the rotary tables stay fp32
        dtype = mat_dtype if (a.ndim == 2 if matrix is None else matrix) else torch.float32
        return torch.from_numpy(a).to(device=dev, dtype=dtype).contiguous()

    jobs = [("tok_emb", -1), ("lm_head", -1), ("final_norm", -1)]
    jobs += [(name, l) for l in range(shape.n_layers) for name in inp.LAYER_TENSORS]
    tensors, layers = {}, [dict() for _ in range(shape.n_layers)]
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        window = 2 * max(1, threads)         # bound the host memory in flight
        for start in range(0, len(jobs), window):
            chunk = jobs[start: start + window]
            futs = [ex.submit(inp.draw_tensor, shape, name, l) for name, l in chunk]
            for (name, l), f in zip(chunk, futs):
                a = f.result()
                t = None if a is None else up(a)
                if l < 0:
                    tensors[name] = t
                else:
                    layers[l][name] = t
    for lt in layers:
        pack_qkv(lt)
    cos, sin = inp.rope_tables(shape, max_seq)
    tensors["rope_cos"], tensors["rope_sin"] = up(cos, matrix=False), up(sin, matrix=False)
    return Model(shape, max_seq, tensors, layers, device)
