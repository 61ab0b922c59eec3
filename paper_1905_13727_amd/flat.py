"""Packing of per-tensor arrays into the library's flat layout and back.
Marshalling only (slicing and copying); no arithmetic of the method."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np


class FlatLayout:
    def __init__(self, plan, shapes: Sequence[tuple]):
        self.shapes = [tuple(int(v) for v in s) for s in shapes]
        self.sizes = plan.sizes
        self.N = int(plan.sizes.n_mat_elems)
        self.L = int(plan.sizes.n_vec_elems)
        self.grad_stride = int(plan.sizes.grad_stride)
        self.flat_off: List[int] = []
        self.p_off: List[int] = []
        self.q_off: List[int] = []
        self.rank: List[int] = []
        self.mat_shape: List[Optional[tuple]] = []
        for t, s in enumerate(self.shapes):
            f, p, q, r = plan.offsets(t)
            self.flat_off.append(f)
            self.p_off.append(p)
            self.q_off.append(q)
            self.rank.append(r)
            if len(s) == 1 or int(np.prod(s[1:])) == 1:
                self.mat_shape.append(None)
            else:
                self.mat_shape.append((s[0], int(np.prod(s[1:]))))

    # flat [N+L]-like buffers -------------------------------------------------
    def pack_flat(self, tensors, length=None, dtype=np.float32, matrices_only=False) -> np.ndarray:
        length = int(length if length is not None else (self.N if matrices_only else self.N + self.L))
        out = np.zeros(length, dtype=dtype)
        for t, a in enumerate(tensors):
            if a is None or (matrices_only and self.mat_shape[t] is None):
                continue
            a = np.asarray(a).reshape(-1)
            out[self.flat_off[t]: self.flat_off[t] + a.size] = a
        return out

    def unpack_flat(self, flat: np.ndarray, matrices_only=False) -> list:
        res = []
        for t, s in enumerate(self.shapes):
            ms = self.mat_shape[t]
            if ms is None:
                res.append(None if matrices_only else
                           np.array(flat[self.flat_off[t]: self.flat_off[t] + s[0]]))
            else:
                n, m = ms
                res.append(np.array(flat[self.flat_off[t]: self.flat_off[t] + n * m]).reshape(n, m))
        return res

    # packed P / Q --------------------------------------------------------------
    def pack_q(self, qs) -> np.ndarray:
        out = np.zeros(int(self.sizes.q_elems), dtype=np.float32)
        for t, q in enumerate(qs):
            if q is None:
                continue
            m, r = self.mat_shape[t][1], self.rank[t]
            assert q.shape == (m, r), (q.shape, m, r)
            out[self.q_off[t]: self.q_off[t] + m * r] = np.asarray(q, dtype=np.float32).reshape(-1)
        return out

    def unpack_q(self, flat: np.ndarray) -> list:
        res = []
        for t in range(len(self.shapes)):
            if self.mat_shape[t] is None:
                res.append(None)
                continue
            m, r = self.mat_shape[t][1], self.rank[t]
            res.append(np.array(flat[self.q_off[t]: self.q_off[t] + m * r]).reshape(m, r))
        return res

    def unpack_p(self, flat: np.ndarray) -> list:
        res = []
        for t in range(len(self.shapes)):
            if self.mat_shape[t] is None:
                res.append(None)
                continue
            n, r = self.mat_shape[t][0], self.rank[t]
            res.append(np.array(flat[self.p_off[t]: self.p_off[t] + n * r]).reshape(n, r))
        return res
