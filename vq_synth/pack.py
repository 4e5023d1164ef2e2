"""Encode-side bit packing of index matrices into the per-row streams the layer stores.

Storage format (one stream per codebook): each output row is its own
little-endian bitstream; index p of the row occupies bits [p*b, (p+1)*b) with
b = ceil(log2 k); bit t of the row is bit (t mod 8) of byte (t div 8); every
row starts on a 16-byte boundary and the pad bits are zero.
"""
import numpy as np


def index_bits(k: int) -> int:
    """Bits per index for a k-entry codebook: ceil(log2 k), at least 1."""
    return max(1, int(k - 1).bit_length())


def row_stride_bytes(per_row: int, bits: int) -> int:
    """Bytes from one row's stream to the next: the row's bits rounded up to 16 bytes."""
    return ((per_row * bits + 127) // 128) * 16


def pack_indices(idx: np.ndarray, bits: int, row_stride: int | None = None) -> np.ndarray:
    """Pack int indices [rows][per_row] into uint8 [rows][row_stride]."""
    idx = np.asarray(idx)
    rows, per_row = idx.shape
    if row_stride is None:
        row_stride = row_stride_bytes(per_row, bits)
    assert row_stride * 8 >= per_row * bits
    if idx.size and (idx.min() < 0 or idx.max() >= (1 << bits)):
        raise ValueError("index does not fit in %d bits" % bits)
    out = np.zeros((rows, row_stride), dtype=np.uint8)
    shifts = np.arange(bits, dtype=np.uint32)
    chunk = max(1, (1 << 24) // max(per_row * bits, 1))
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        part = idx[r0:r1].astype(np.uint32)
        bitplane = ((part[:, :, None] >> shifts) & 1).astype(np.uint8).reshape(r1 - r0, per_row * bits)
        packed = np.packbits(bitplane, axis=1, bitorder="little")
        out[r0:r1, : packed.shape[1]] = packed
    return out
