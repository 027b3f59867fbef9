"""Helpers of the GPU parity tests: numpy <-> device tensor marshalling and the comparison rules."""
import numpy as np
import torch


def to_bf16_dev(bits: np.ndarray):
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on the GPU (bit-preserving)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bf16_bits(t) -> np.ndarray:
    """torch.bfloat16 tensor (any device) -> uint16 bit patterns on the host."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def dev(a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def with_poisoned_tail(t, slack: int = 65536):
    """The device tensor t re-allocated as the front of a larger buffer whose tail holds 0xFF bytes (NaN as bf16 /
    fp32, -1 as int32): a kernel that reads a little past the end of t stays inside the allocation, and if the value
    read takes part in a result the result turns NaN or fails its comparison."""
    flat = t.contiguous().view(torch.uint8).reshape(-1)
    big = torch.full((flat.numel() + slack,), 0xFF, dtype=torch.uint8, device=t.device)
    big[:flat.numel()] = flat
    return big[:flat.numel()].view(t.dtype).reshape(t.shape)


def host(t) -> np.ndarray:
    return t.detach().cpu().numpy()


def row_rel_err(y, y_ref):
    """Per token row: max_h |y - y_ref| / max_h |y_ref| (the layer-output tolerance is stated on this)."""
    y = np.asarray(y, np.float64)
    y_ref = np.asarray(y_ref, np.float64)
    den = np.abs(y_ref).max(axis=1)
    den = np.where(den == 0, 1.0, den)
    return np.abs(y - y_ref).max(axis=1) / den


def pack_reference(W: np.ndarray) -> np.ndarray:
    """Row-major [E,R,K] -> [E,R/16,K/32,64,8]: entry (lane l, i) = W[rt*16 + l%16][kt*32 + (l//16)*8 + i]."""
    E, R, K = W.shape
    t = W.reshape(E, R // 16, 16, K // 32, 4, 8)       # e, rt, r, kt, g, i
    return np.ascontiguousarray(t.transpose(0, 1, 3, 4, 2, 5)).reshape(E, R // 16, K // 32, 64, 8)   # lane = g*16 + r


def tile_covering_tokens(offsets, perm, k):
    """Tokens that between them sit in every 16-token column tile of three experts: the fullest one that streams
    without the LDS stage (at most 16 tokens), the fullest one of 17 to 64 tokens (a 64-token pass) and the fullest
    one beyond 64 (128-token passes), where the batch has such experts.  A fault tied to a position inside an expert's
    token range, e.g. one column tile of a pass, cannot hide between random samples."""
    te = np.diff(offsets)
    picked = []
    for lo, hi in ((1, 16), (17, 64), (65, 1 << 30)):
        cand = np.flatnonzero((te >= lo) & (te <= hi))
        if cand.size == 0:
            continue
        e = int(cand[np.argmax(te[cand])])
        for tile in range((int(te[e]) + 15) // 16):
            pos = offsets[e] + min(16 * tile + (5 * tile + 3) % 16, int(te[e]) - 1)   # a different lane in every tile
            picked.append(int(perm[pos]) // k)
    return picked
