"""Small host-side helpers shared by the tests (no method arithmetic)."""
import numpy as np
import torch


def to_bf16_bits(x) -> np.ndarray:
    """float array -> bf16 bit patterns (uint16), round-to-nearest-even."""
    t = torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def logits_from_probs(p) -> np.ndarray:
    """fp32 logits whose softmax is p (up to fp32 rounding of ln p)."""
    return np.log(np.asarray(p, dtype=np.float64)).astype(np.float32)


def read_golden(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            rows.append([c.strip() for c in line.split("|")])
    return rows
