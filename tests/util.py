"""Helpers shared by the tests (no method arithmetic of the product or the oracle)."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            parts = line.split()
            out[parts[0]] = parts[1:] if len(parts) > 2 else parts[1]
    return out


def storage_order_view(W):
    """The documented element order of the format, written with numpy reshapes only:
    returns W as [n_bt, tt(8), ft(8), p(64)] where BlockTiles run K-fastest inside a
    64-row strip, TensorCoreTiles (16 x 32) and FragTiles (8 x 8) run N-fastest inside
    their parent, and p = 8 * row + col."""
    N, K = W.shape
    v = W.reshape(N // 64, 4, 2, 8, K // 64, 2, 4, 8)
    #             strip  ttn ftn r   kb      ttk ftk c
    v = v.transpose(0, 4, 5, 1, 6, 2, 3, 7)
    #               strip kb ttk ttn ftk ftn r c
    return np.ascontiguousarray(v).reshape((N // 64) * (K // 64), 8, 8, 64)
