"""Helpers shared by the GPU parity tests (no arithmetic of the method)."""
import numpy as np

from oracle import layer as L
from paper_2204_12013_amd import synth

TOL = {synth.DTYPE_FP32: 1e-4, synth.DTYPE_BF16: 2e-2}


def rel_l2(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    denom = np.linalg.norm(want.ravel())
    return float(np.linalg.norm((got - want).ravel()) / (denom if denom > 0 else 1.0))


def oracle_layers(flat_layers, H, F):
    """[n, layer_params] float32 -> list of named float64 parameter dicts."""
    return [L.unpack_layer(np.asarray(row, dtype=np.float64), H, F) for row in flat_layers]


def check_grads(got_flat, want_named_list, H, F, tol, label):
    """Per named tensor per layer relative L2 (not one global norm)."""
    got_flat = np.asarray(got_flat, dtype=np.float64).reshape(len(want_named_list), -1)
    worst = 0.0
    for l, want in enumerate(want_named_list):
        got = L.unpack_layer(got_flat[l], H, F)
        for n in L.PARAM_NAMES:
            e = rel_l2(got[n], want[n])
            worst = max(worst, e)
            assert e <= tol, "%s layer %d %s: rel L2 %.3e > %.1e" % (label, l, n, e, tol)
    return worst
