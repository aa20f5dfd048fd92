"""MI355X-native hot path of Parallel Speculative Decoding (PSD) for masked-diffusion LLMs.

Thin ctypes binding over libpsd.so (see include/psd.h).  Argument marshalling only: every
step of the path runs in the HIP kernels of the library.  PyTorch provides device memory
and the stream.
"""
from .binding import (Model, Policy, Graph, Stats, PsdError, load_library, library_path, chain_graph,
                      psd_forward_confidence, psd_forward_logits, psd_select_unmask, psd_build_drafts,
                      psd_accept, psd_verify_accept, psd_decode_block, psd_decode, decode, forward_work, KvCache, psd_kv_prefill,
                      psd_forward_confidence_cached, psd_decode_block_cached, lattice_graph, psd_calibrate_graph,
                      psd_forward_confidence_approx, psd_decode_block_approx)

__all__ = ["Model", "Policy", "Graph", "Stats", "PsdError", "load_library", "library_path", "chain_graph",
           "psd_forward_confidence", "psd_forward_logits", "psd_select_unmask", "psd_build_drafts", "psd_accept",
           "psd_verify_accept", "psd_decode_block", "psd_decode", "decode", "forward_work", "KvCache", "psd_kv_prefill",
           "psd_forward_confidence_cached", "psd_decode_block_cached", "lattice_graph", "psd_calibrate_graph", "psd_forward_confidence_approx",
           "psd_decode_block_approx"]
