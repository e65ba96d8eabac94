"""Exit statistics reported alongside the router outputs (paper Table 1 "Distribution"
column, Fig. 3's layer-ops count).  Host-side bookkeeping on the exit_layer array."""
from __future__ import annotations

import numpy as np


def exit_histogram(exit_layer, layer_ids, no_exit_layer) -> dict:
    """{'L11': 16, 'L31': 306, ...} in the style of Table 1, plus 'none' for no early exit."""
    ex = np.asarray(exit_layer)
    out = {f"L{int(l)}": int((ex == l).sum()) for l in layer_ids if (ex == l).any()}
    n_none = int((ex == no_exit_layer).sum())
    if n_none:
        out["none"] = n_none
    return out


def exit_rate(exit_layer, no_exit_layer) -> float:
    ex = np.asarray(exit_layer)
    return float((ex != no_exit_layer).mean()) if ex.size else 0.0


def layer_ops(exit_layer, n_layers: int) -> tuple[int, int, float]:
    """(layer-ops with exits, without, fraction saved), counting as Fig. 3 does: a token
    that exits at layer k costs k layer-ops, one that never exits costs n_layers."""
    ex = np.minimum(np.asarray(exit_layer, dtype=np.int64), n_layers)
    used, full = int(ex.sum()), int(ex.size) * int(n_layers)
    return used, full, (1.0 - used / full) if full else 0.0
