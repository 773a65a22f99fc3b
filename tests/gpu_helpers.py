"""Shared plumbing of the GPU parity tests: upload seeded inputs, build expert
tables, error metrics.  Holds no arithmetic of the method."""
import numpy as np
import torch

from oracle import dymoe_oracle as O
from paper_2603_19172_amd import binding as B
from paper_2603_19172_amd import synth

DEV = "cuda:0"


def to_bf16(bits_u16: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).to(DEV).view(torch.bfloat16)


def to_f16(bits_u16: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).to(DEV).view(torch.float16)


def bits_of(t: torch.Tensor) -> np.ndarray:
    """16-bit tensor -> uint16 bit patterns on the host."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def oracle_quantize_expert(mats, bits):
    return [O.quantize_pack(m, bits) for m in mats]


def upload_q(trip):
    return [(torch.from_numpy(cd).to(DEV), to_f16(sc), to_f16(zr)) for cd, sc, zr in trip]


def empty_q(F, H, bits):
    out = []
    for (n, k) in ((F, H), (F, H), (H, F)):
        out.append((torch.empty((n, k * bits // 8), dtype=torch.uint8, device=DEV),
                    torch.empty((n, k // 64), dtype=torch.float16, device=DEV),
                    torch.empty((n, k // 64), dtype=torch.float16, device=DEV)))
    return out


def tiles_from_rowmajor(codes, scale, zero, bits):
    """Row-major packed matrix -> the library's 32x128 tile layout (a pure
    permutation of bytes; see include/dymoe.h)."""
    N = codes.shape[0]
    K = codes.shape[1] * 8 // bits
    NT, KT = N // 32, K // 128
    C = bits // 2     # 16-byte chunks per lane; row bytes: (kt, kb, c, 16) -> tile (c, kb, r, 16)
    t = codes.reshape(NT, 32, KT, 2, C, 16).transpose(0, 2, 4, 3, 1, 5)
    sz = lambda a: np.ascontiguousarray(a.reshape(NT, 32, KT, 2).transpose(0, 2, 3, 1)).reshape(N, K // 64)
    return np.ascontiguousarray(t).reshape(codes.shape), sz(scale), sz(zero)


def rowmajor_from_tiles(codes, scale, zero, bits):
    N = codes.shape[0]
    K = codes.shape[1] * 8 // bits
    NT, KT = N // 32, K // 128
    C = bits // 2
    t = codes.reshape(NT, KT, C, 2, 32, 16).transpose(0, 4, 1, 3, 2, 5)
    sz = lambda a: np.ascontiguousarray(a.reshape(NT, KT, 2, 32).transpose(0, 3, 1, 2)).reshape(N, K // 64)
    return np.ascontiguousarray(t).reshape(codes.shape), sz(scale), sz(zero)


def bf16_tiles_from_rowmajor(w):
    """bf16 bit patterns [N,K] -> tile layout: row elements (kt, kb, j, 8) -> tile (j, kb, r, 8)."""
    N, K = w.shape
    NT, KT = N // 32, K // 128
    t = w.reshape(NT, 32, KT, 2, 8, 8).transpose(0, 2, 4, 3, 1, 5)
    return np.ascontiguousarray(t).reshape(N, K)


def rel_err_per_token(y: np.ndarray, ref: np.ndarray) -> float:
    """max over tokens of max_j |y - ref| / rms_j(ref[t])."""
    rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
    rms = np.where(rms > 0, rms, 1.0)
    return float((np.abs(y - ref) / rms).max())


def margin_ok(logits: np.ndarray, k: int, tol: float = 1e-4) -> np.ndarray:
    """Per token: every adjacent pair among the k+1 largest logits differs by > tol."""
    s = -np.sort(-logits, axis=1)[:, :min(k + 1, logits.shape[1])]
    return (s[:, :-1] - s[:, 1:] > tol).all(axis=1)
