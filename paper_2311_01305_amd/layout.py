"""Index permutations between a row-major int8 matrix and the K-panel layout of the GEMM
operands (64-column panels, rows back to back inside a panel, zero fill past K).  Host-side
marshalling for callers that inspect or supply codes; the device converters are
aweq_pack_panels_i8 / aweq_unpack_panels_i8."""
import numpy as np

PANEL = 64


def to_panels(mat: np.ndarray) -> np.ndarray:
    rows, K = mat.shape
    kp = -(-K // PANEL)
    padded = np.zeros((rows, kp * PANEL), dtype=mat.dtype)
    padded[:, :K] = mat
    return np.ascontiguousarray(padded.reshape(rows, kp, PANEL).transpose(1, 0, 2)).reshape(-1)


def from_panels(buf: np.ndarray, rows: int, K: int) -> np.ndarray:
    kp = -(-K // PANEL)
    a = np.asarray(buf).reshape(-1)[:kp * rows * PANEL].reshape(kp, rows, PANEL).transpose(1, 0, 2)
    return np.ascontiguousarray(a.reshape(rows, kp * PANEL)[:, :K])
