"""CPU oracle for the mask generator of the sparse-training pipeline (TEST INFRASTRUCTURE ONLY).

Only ``tests/`` and ``__graft_entry__.smoke()`` may import this module; it imports nothing from the
HIP package and shares no code with it.  Plain numpy, written for checking by eye.

What it computes -- Alg. 1, function getMask (Sec. 3.1 describes it in words):

  1. a random 2-D score at the resolution of the network input is GIVEN (the random numbers are an
     input of the oracle and of the GPU path alike);
  2. for every layer, ``ratio = input_res // layer_res`` and the layer's score is the average pooling
     of the input score with window = stride = ratio (no padding);
  3. the pixels of the layer are ranked by that score and the mask is all ones except at the ranked
     pixels that are dropped, which are set to 0.

Readings taken where the algorithm is silent:

  * the ratio is taken per axis (``in_h // ho`` and ``in_w // wo``) so non-square maps work; when the
    pooled map is larger than the layer (resolution not divisible) its top-left ``ho x wo`` corner is
    used;
  * the rank key of a pixel is the SUM of its pooling window, accumulated in double precision in
    row-major order of the window starting from +0.0.  Dividing every sum by the same window size
    orders the pixels identically, and leaving the division out keeps a rounding step from merging
    two different sums into a tie;
  * the pixels with the LOWEST keys are dropped, ``n - kept`` of them with
    ``kept = floor((1 - s) * n + 0.5)`` (the kept-row count of Sec. 3.2), equal keys in ascending
    pixel index (row-major);
  * one mask per layer resolution, shared by the whole batch and all channels (Sec. 3: the mask is 2-D).
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np


def kept_pixels(sparsity: float, n: int) -> int:
    """Pixels a layer keeps: n - s*n rounded half up (Sec. 3.2)."""
    return int(math.floor((1.0 - float(sparsity)) * n + 0.5))


def layer_score_sums(score: np.ndarray, ho: int, wo: int) -> np.ndarray:
    """Window sums (double) of the average pooling of Alg. 1 for a layer of resolution ho x wo."""
    score = np.asarray(score)
    assert score.ndim == 2 and score.dtype == np.float32
    in_h, in_w = score.shape
    assert 1 <= ho <= in_h and 1 <= wo <= in_w
    rh, rw = in_h // ho, in_w // wo
    sums = np.zeros((ho, wo), dtype=np.float64)
    for oy in range(ho):
        for ox in range(wo):
            acc = 0.0
            for dy in range(rh):
                for dx in range(rw):
                    acc = acc + float(score[oy * rh + dy, ox * rw + dx])
            sums[oy, ox] = acc
    return sums


def rank_pixels(keys: np.ndarray, n_drop: int) -> np.ndarray:
    """Indices (row-major) of the n_drop pixels with the lowest keys, equal keys by lower index."""
    flat = np.asarray(keys, dtype=np.float64).reshape(-1)
    order = np.argsort(flat, kind="stable")          # ascending, ties keep index order
    return order[:n_drop]


def layer_mask(score: np.ndarray, ho: int, wo: int, sparsity: float) -> np.ndarray:
    """uint8 mask [ho, wo] of one layer: 1 = keep, 0 = drop."""
    n = ho * wo
    n_drop = n - kept_pixels(sparsity, n)
    idx = rank_pixels(layer_score_sums(score, ho, wo), n_drop)
    mask = np.ones(n, dtype=np.uint8)
    mask[idx] = 0
    return mask.reshape(ho, wo)


def get_mask(score: np.ndarray, layer_resolutions: Sequence[Tuple[int, int]], sparsity) -> List[np.ndarray]:
    """Alg. 1 getMask: one mask per layer from one input-resolution score.  `sparsity` is a number or
    one number per layer."""
    if np.isscalar(sparsity):
        sparsity = [float(sparsity)] * len(layer_resolutions)
    assert len(sparsity) == len(layer_resolutions)
    return [layer_mask(score, ho, wo, s) for (ho, wo), s in zip(layer_resolutions, sparsity)]
