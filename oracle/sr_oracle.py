"""CPU oracle for the shared/residual (SR) expert compression.

TEST INFRASTRUCTURE ONLY.  Slow, plain reference for the SREncode / SRDecode kernels; only
tests, the smoke check and the benchmark's `cpu_baseline` leg may import it.  It shares no
code with the HIP kernels and does not import the GPU package.

What the paper fixes (Sec. 4.2 "SR-Based Expert Compression", Fig. "SRexpert"(b)):

  encode  residual = expert - shared expert; the residual is compressed by Top-k and kept
          in value-index form for the transfer;
  decode  the compressed residual is recovered and added to the shared expert, the two
          steps fused;
  CR      the compression ratio is the hyper-parameter (50 in the paper's experiments,
          Sec. 5.4 "Configurations of SR-Based Expert Compression").

Readings taken where the paper is silent (listed again in the design notes):

  * Top-k is by magnitude |residual| (a Top-k of signed values would drop every negative
    correction; the paper's naive baseline "directly compresses the expert through Top-k"
    only makes sense by magnitude as well);
  * k = floor(n / CR), at least 1, n = number of elements of the weight matrix;
  * equal magnitudes: the lower flat index is kept first;
  * the value-index list is ordered by ascending index;
  * precision: the residual is the float32 difference of the stored values and that float32
    number decides the selection (the paper fixes no precision; a selection is an integer
    decision, so oracle and kernel take it in the same, the kernel's, precision); the
    transmitted value is the residual rounded to the storage type (round to nearest even);
    decode adds in float32 and rounds once to the storage type.

Storage types: "f32" (numpy float32) and "bf16" (uint16 bit patterns), as everywhere in
this repository.

Pins (tests/test_oracle_sr.py): brute-force selection in pure Python, torch.topk /
numpy.argpartition on distinct magnitudes, the special cases shared = 0 (plain Top-k
sparsification) and k = n, planted ties, the invariants "kept >= dropped", "dropped
positions decode to the shared expert exactly", the rounding against torch's
float32 -> bfloat16 conversion.  No function here is "parity unpinned".
"""
from __future__ import annotations

from typing import Tuple

import numpy as np

F32 = np.float32


# ------------------------------------------------------------------ storage
def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact: a bf16 pattern is the upper half of a float32."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(F32)


def f32_to_bf16_rne(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern, round to nearest, ties to even (no NaN inputs)."""
    u = np.ascontiguousarray(x, dtype=F32).view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    return ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)


def to_f32(stored: np.ndarray, storage: str) -> np.ndarray:
    return bf16_to_f32(stored) if storage == "bf16" else stored.astype(F32)


def to_storage(x: np.ndarray, storage: str) -> np.ndarray:
    return f32_to_bf16_rne(x) if storage == "bf16" else x.astype(F32)


# ------------------------------------------------------------------ the method
def keep_count(n: int, cr: int) -> int:
    """Entries kept for compression ratio CR (Sec. 5.4): floor(n / CR), at least one."""
    return max(1, n // cr)


def residual(expert: np.ndarray, shared: np.ndarray, storage: str) -> np.ndarray:
    """Encode, first step (Sec. 4.2): expert minus shared expert, in float32."""
    return to_f32(expert.ravel(), storage) - to_f32(shared.ravel(), storage)


def select_topk(res: np.ndarray, k: int) -> np.ndarray:
    """Encode, second step: the k entries of largest magnitude; among equal magnitudes the
    lower index first.  Returns their flat indices in ascending order."""
    mag = np.abs(res)
    n = mag.shape[0]
    order = np.lexsort((np.arange(n), -mag))  # last key is primary: magnitude descending
    return np.sort(order[:k]).astype(np.int32)


def sr_encode(expert: np.ndarray, shared: np.ndarray, k: int,
              storage: str) -> Tuple[np.ndarray, np.ndarray]:
    """SREncode (Sec. 4.2): value-index form of the Top-k residual."""
    res = residual(expert, shared, storage)
    idx = select_topk(res, k)
    return to_storage(res[idx], storage), idx


def sr_decode(shared: np.ndarray, values: np.ndarray, indices: np.ndarray,
              storage: str) -> np.ndarray:
    """SRDecode (Sec. 4.2), both steps at once: shared expert plus the scattered residual."""
    out = to_f32(shared.ravel(), storage).copy()
    out[indices] = out[indices] + to_f32(values, storage)
    return to_storage(out, storage).reshape(shared.shape)
