"""numpy reader / writer of the packed-cache bit layouts documented in
include/zipcache.h (ROW for keys, TGROUP for values).  Written from the
header's description only, so that the tests check the bytes the kernels
produce rather than trusting a kernel to unpack them."""
import numpy as np


def _tile_of_field_group(bits: int, jf: int) -> int:
    return (0, 2, 1, 3)[jf] if bits == 2 else jf


def decode_row(arena: np.ndarray, B: int, H: int, D: int, cap: int, bits: int) -> np.ndarray:
    """uint8 arena -> codes [B, H, cap, D]."""
    a = np.asarray(arena, np.uint8)[: B * H * cap * D * bits // 8].reshape(B, H, cap, D * bits // 8)
    b = np.unpackbits(a, axis=-1, bitorder="little").reshape(B, H, cap, D, bits)
    return (b.astype(np.int64) << np.arange(bits)).sum(-1)


def encode_row(codes: np.ndarray, bits: int) -> np.ndarray:
    """codes [B, H, cap, D] -> uint8 arena (flat)."""
    c = np.asarray(codes, np.int64)
    b = ((c[..., None] >> np.arange(bits)) & 1).astype(np.uint8)
    B, H, cap, D = c.shape
    return np.packbits(b.reshape(B, H, cap, D * bits), axis=-1, bitorder="little").reshape(-1)


def decode_tgroup(arena: np.ndarray, B: int, H: int, D: int, cap: int, bits: int) -> np.ndarray:
    """uint8 arena -> codes [B, H, cap, D]."""
    E = 32 // bits
    TB = 4 * E
    nblk = cap // TB
    w = np.asarray(arena, np.uint8)[: B * H * cap * D * bits // 8].view(np.uint32).reshape(B, H, nblk, 4, D)
    out = np.zeros((B, H, nblk, TB, D), np.int64)
    mask = (1 << bits) - 1
    for e in range(E):
        field = (w >> np.uint32(bits * e)) & np.uint32(mask)
        j = _tile_of_field_group(bits, e // 4)
        for kg in range(4):
            out[:, :, :, 16 * j + 4 * kg + e % 4, :] = field[:, :, :, kg, :]
    return out.reshape(B, H, cap, D)


def encode_tgroup(codes: np.ndarray, bits: int) -> np.ndarray:
    """codes [B, H, cap, D] (cap a multiple of the block size) -> uint8 arena."""
    c = np.asarray(codes, np.int64)
    B, H, cap, D = c.shape
    E = 32 // bits
    TB = 4 * E
    nblk = cap // TB
    c = c.reshape(B, H, nblk, TB, D)
    w = np.zeros((B, H, nblk, 4, D), np.uint32)
    for e in range(E):
        j = _tile_of_field_group(bits, e // 4)
        for kg in range(4):
            w[:, :, :, kg, :] |= (c[:, :, :, 16 * j + 4 * kg + e % 4, :].astype(np.uint32) << np.uint32(bits * e))
    return w.reshape(-1).view(np.uint8)


def to_token_rows(codes_bhsd: np.ndarray) -> np.ndarray:
    """[B, H, slots, D] -> [B, slots, H*D] (channel index = head*D + c)."""
    B, H, S, D = codes_bhsd.shape
    return codes_bhsd.transpose(0, 2, 1, 3).reshape(B, S, H * D)


def from_token_rows(rows: np.ndarray, H: int) -> np.ndarray:
    B, S, W = rows.shape
    return rows.reshape(B, S, H, W // H).transpose(0, 2, 1, 3)
