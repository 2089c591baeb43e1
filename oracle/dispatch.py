"""TEST INFRASTRUCTURE -- oracle of the Dispatch step (section 3.2: the rules that prepare the tasks' inputs for the
batched BaseOp; section 3.5: where each token sits in the chunk-aligned batch).

Every task hands over its tokens densely packed, [valid_t, width]: its sequences one after the other in the order of
its sequence list.  In the aligned batch the task's tokens occupy its valid rows in ascending order (packing and
chunking keep the order of the tokens), and every other row is padding, which is zero.  Written with the row -> task
map of the oracle's own table (oracle/segtab.py); no arithmetic, only placement."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np


def gather(task_inputs: Sequence[Optional[np.ndarray]], row_task: np.ndarray, width: int) -> np.ndarray:
    """Per-task packed inputs -> aligned batch [T, width]."""
    T = len(row_task)
    X = np.zeros((T, width), dtype=np.float64)
    for t, src in enumerate(task_inputs):
        rows = np.nonzero(row_task == t)[0]
        if len(rows):
            src = np.asarray(src, dtype=np.float64)
            assert src.shape == (len(rows), width)
            X[rows] = src
    return X


def scatter(X: np.ndarray, row_task: np.ndarray, n_tasks: int) -> List[np.ndarray]:
    """Aligned batch -> per-task packed outputs (padding rows are dropped)."""
    X = np.asarray(X, dtype=np.float64)
    return [X[np.nonzero(row_task == t)[0]] for t in range(n_tasks)]
