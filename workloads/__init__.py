"""Seeded synthetic inputs for the FreeKV retrieval-decode path.

This package only *produces* tensors (keys, values, queries) and names the
workload shapes.  It holds none of the method's arithmetic: no page summaries,
no scores, no selection, no attention.  Both the CPU oracle's tests and the
HIP path's tests/bench draw their inputs from here so that the two sides see
byte-identical data without sharing any code of the method itself.
"""
from .configs import Workload, WORKLOADS, get_workload
from .synth import (
    encode, decode, kv_prefix, kv_decode_tokens, query_stream, OUTLIER_CHANNELS,
)

__all__ = [
    "Workload", "WORKLOADS", "get_workload", "encode", "decode", "kv_prefix",
    "kv_decode_tokens", "query_stream", "OUTLIER_CHANNELS",
]
