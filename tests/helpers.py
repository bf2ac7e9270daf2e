"""Glue used by the tests only."""
from __future__ import annotations

import numpy as np

from oracle.harness import F64Weights, oracle_model, oracle_requests  # noqa: F401
from paper_2506_09397_amd import synth


def split_rows(batch: synth.Batch, arr: np.ndarray):
    offs = batch.row_offsets()
    return [arr[offs[i]: offs[i + 1]] for i in range(batch.B)]
