"""Shared fixtures for the GPU parity tests (HIP path through the C ABI vs the CPU oracle)."""
import sys

import numpy as np


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def to_u64(t):
    """torch int64 tensor of mask words -> numpy uint64."""
    return t.cpu().numpy().view(np.uint64)


def make_context(w, biases=None, transform_dtype=0):
    from paper_2506_22668_amd import Context
    ctx = Context("cuda:0")
    ctx.set_graph(w.row_ptr, w.col)
    ctx.set_features(w.features)
    ctx.set_gcn(w.weights, biases=biases, transform_dtype=transform_dtype)
    return ctx
