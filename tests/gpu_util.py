"""Helpers shared by the GPU parity tests (marshalling between torch and the numpy oracle)."""
import numpy as np
import torch

import oracle as O


def to_np(t):
    """GPU/CPU torch tensor -> numpy array the oracle accepts (bf16 as uint16 bit patterns)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def ofmt(f):
    """Library format -> oracle format (same six integers, separately declared types)."""
    return O.Format(f.k1, f.d1, f.k2, f.d2, f.m, f.rounding)


def assert_planes_equal(got, want, what=""):
    for name, g, w in zip(("codes", "sexp", "mexp"), got, want):
        g = g.cpu().numpy()
        assert g.shape == w.shape, (what, name, g.shape, w.shape)
        if not np.array_equal(g, w):
            bad = np.flatnonzero(g != w)
            raise AssertionError("%s %s: %d of %d bytes differ, first at byte %d (got %d want %d)"
                                 % (what, name, bad.size, g.size, bad[0], g[bad[0]], w[bad[0]]))


def assert_bits_equal(got, want, what=""):
    g, w = to_np(got), np.asarray(want)
    gi = g.view(np.uint32) if g.dtype == np.float32 else g
    wi = w.view(np.uint32) if w.dtype == np.float32 else w
    assert gi.shape == wi.shape, (what, gi.shape, wi.shape)
    if not np.array_equal(gi, wi):
        bad = np.flatnonzero(gi.reshape(-1) != wi.reshape(-1))
        i = bad[0]
        raise AssertionError("%s: %d of %d values differ, first at %d (got %r want %r)"
                             % (what, bad.size, gi.size, i, g.reshape(-1)[i], w.reshape(-1)[i]))
