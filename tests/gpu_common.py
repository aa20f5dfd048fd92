"""Helpers shared by the GPU parity tests (imported only from tests marked gpu)."""
import numpy as np
import torch

import psd_inputs as inp
import paper_2605_15609_amd as psd
from oracle import psd_oracle as orc

DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


def to_dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return t if dtype is None else t.to(dtype)


def oracle_graph(g: "psd.Graph") -> orc.Graph:
    return orc.Graph(tuple(frozenset(r for r in range(64) if (bits >> r) & 1) for bits in g.rank_sets))


def gpu_graph(g: orc.Graph) -> "psd.Graph":
    return psd.Graph(tuple(sum(1 << r for r in ranks) for ranks in g.rank_sets))


def make_models(shape, max_seq):
    host = inp.draw_model(shape, max_seq)
    return host, psd.Model.from_host(host, DEV)
