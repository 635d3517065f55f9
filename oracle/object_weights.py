"""CPU oracle of the loss-weight map (Section 5.2: the cross-entropy of pixels near and within
non-background objects is scaled by a factor of 5).

TEST INFRASTRUCTURE.  Only tests/, the smoke check and the benchmark's cpu_baseline leg may
import this module; the product (paper_2003_10735_amd) never does.

The paper gives the factor and leaves "near" open.  The reading taken here: a pixel is near an
object when some pixel of the same frame at most `radius` columns and at most `radius` rows away
carries an object label (a square neighbourhood, cut off at the frame's edges).  A label is an
object when it is a class index in [0, n_classes) other than `background` and `ignore_index`.
The map holds `factor` on every such pixel and 1 on every other one.

Written as that definition: for every offset (dy, dx) of the neighbourhood, every pixel whose
neighbour at that offset is an object is marked.  No separable passes, no distance transform.
"""
from __future__ import annotations

import numpy as np


def is_object(labels: np.ndarray, n_classes: int, background: int, ignore_index: int) -> np.ndarray:
    lab = np.asarray(labels)
    return (lab >= 0) & (lab < n_classes) & (lab != background) & (lab != ignore_index)


def object_weights(labels: np.ndarray, n_classes: int, radius: int, factor: int = 5, background: int = 0,
                   ignore_index: int = -1) -> np.ndarray:
    """labels [n, H, W] integer -> weights [n, H, W] uint8."""
    lab = np.asarray(labels)
    assert lab.ndim == 3 and radius >= 0 and 1 <= factor <= 255
    _, H, W = lab.shape
    obj = is_object(lab, n_classes, background, ignore_index)
    near = np.zeros_like(obj)
    for dy in range(-radius, radius + 1):
        for dx in range(-radius, radius + 1):
            # pixel (y, x) looks at (y + dy, x + dx); both must lie inside the frame
            ya, yb = max(0, -dy), min(H, H - dy)
            xa, xb = max(0, -dx), min(W, W - dx)
            if ya >= yb or xa >= xb:
                continue
            near[:, ya:yb, xa:xb] |= obj[:, ya + dy:yb + dy, xa + dx:xb + dx]
    return np.where(near, factor, 1).astype(np.uint8)
