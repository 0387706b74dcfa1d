"""Shared helpers of the GPU parity tests (no method arithmetic here)."""
import numpy as np
import torch

import workloads


def make_ctx(model, weights_cpu, **kw):
    from paper_2605_26606_amd import Context
    wd = workloads.weights_to(weights_cpu, "cuda")
    return Context(model, wd, **kw)


def side_stream():
    return torch.cuda.Stream()


def say(msg):
    print("[gpu-test] " + msg, flush=True)
