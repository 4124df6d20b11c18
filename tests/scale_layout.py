"""Test-side index maps between the two scale layouts of include/mxfp8.h (numpy, no arithmetic on
the values): row-major s[r, b] and tiled s[((r//64 * ceil(nb/4) + b//4) * 64 + r%64) * 4 + b%4]."""
import numpy as np


def tiled_bytes(rows, nb):
    return ((rows + 63) // 64) * ((nb + 3) // 4) * 256


def _index(rows, nb):
    r = np.arange(rows)[:, None]
    b = np.arange(nb)[None, :]
    return ((r // 64 * ((nb + 3) // 4) + b // 4) * 64 + r % 64) * 4 + b % 4


def tile(s, filler=0xEE):
    """[rows x nb] -> flat tiled buffer; positions without a (row, block) hold `filler`."""
    rows, nb = s.shape
    out = np.full(tiled_bytes(rows, nb), filler, np.uint8)
    out[_index(rows, nb)] = s
    return out


def untile(flat, rows, nb):
    """flat tiled buffer -> [rows x nb]."""
    flat = np.asarray(flat).reshape(-1)
    assert flat.size >= tiled_bytes(rows, nb)
    return flat[_index(rows, nb)]


def filler_mask(rows, nb):
    """True at the bytes of a tiled buffer that belong to no (row, block)."""
    m = np.ones(tiled_bytes(rows, nb), bool)
    m[_index(rows, nb)] = False
    return m
