"""Helpers for the GPU parity tests: one context per session, numpy <-> device."""
import numpy as np

_ctx = None


def ctx():
    global _ctx
    if _ctx is None:
        from paper_2110_03423_amd import Rsvd
        _ctx = Rsvd(0)
    return _ctx


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def to_np(t):
    return t.detach().cpu().numpy()


def say(*args):
    print(*args, flush=True)
