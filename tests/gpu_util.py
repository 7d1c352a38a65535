"""Helpers for the GPU parity tests: move byte arrays to and from the device."""
import numpy as np
import torch

import kvl_workloads as W
import paper_2602_21548_amd as K


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a).to("cuda")


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy()


def planes_to_dev(planes):
    return [to_dev(p) for p in planes]


def dev_plan(w, side, flags, **tuning):
    s = w.src if side == "src" else w.dst
    lay = K.make_layout(w.layout.n_layers, w.layout.block_tokens, w.layout.row_bytes, s.pool_blocks)
    return K.kvl_plan(lay, w.hit, w.app, s.tables, flags, **tuning)


def same_bytes(a: np.ndarray, b: np.ndarray) -> bool:
    return a.shape == b.shape and a.tobytes() == b.tobytes() if a.size < (1 << 28) else np.array_equal(a, b)


def pinned_from(a: np.ndarray) -> torch.Tensor:
    t = torch.empty(a.size, dtype=torch.uint8, pin_memory=True)
    t.numpy()[:] = a
    return t
