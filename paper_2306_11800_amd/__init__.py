"""MI355X-native hot path of the checkpoint compressor: search, quantize, delta.

The work is done by HIP kernels behind the C ABI of include/inshr.h (libinshr.so); this package only
marshals arguments.  `synth` holds the seeded input generators used by tests and bench."""
from . import synth  # noqa: F401


def Context(*args, **kwargs):
    """inshr_create: see api.Context."""
    from .api import Context as _C
    return _C(*args, **kwargs)


def inshr_search(ctx, tensors, grid, eps, want_scores=True):
    return ctx.search(tensors, grid, eps, want_scores)


def inshr_quantize(ctx, tensors, cfgs, reuse_search=False, out=None):
    return ctx.quantize(tensors, cfgs, reuse_search, out)


def inshr_delta(ctx, prev, cur, want_perm=False, prev_perm=None, out=None):
    return ctx.delta(prev, cur, want_perm, prev_perm, out)
