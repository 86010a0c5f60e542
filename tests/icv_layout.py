"""Test-side decoding of the indirection buffer, from what icv_get_indirection_layout reports.

The library stores entries in the order and width its kernels read best; the tests compare their meaning
(output pixel, kernel element) -> input pixel or zero row with the oracle's, so everything here is undoing the
physical layout on the host.
"""
import numpy as np

from paper_1907_02129_amd import binding as icv

_ESZ = {icv.ICV_F32: 4, icv.ICV_BF16: 2, icv.ICV_U8I8: 1}


def _stride_bytes(p) -> int:
    return (p.in_pixel_stride or p.C) * _ESZ[p.dtype]


def tile_records(p, indirection):
    """(records (tiles, 4) int32, 2-byte entries (tiles, T, tile_rows) uint16), or None when the plan reads int32 entries."""
    L = icv.get_indirection_layout(p)
    if L.entry_bytes != 2:
        return None
    T = p.R * p.S
    raw = indirection.cpu().numpy().view(np.uint8)
    assert L.record_bytes == 16 and L.records_at >= 0
    rec = raw[L.records_at:L.records_at + L.tiles * 16].view(np.int32).reshape(L.tiles, 4)
    n = L.tiles * T * L.tile_rows
    ent = raw[L.entries_at:L.entries_at + 2 * n].view(np.uint16).reshape(L.tiles, T, L.tile_rows)
    return rec, ent


def logical_indirection(p, indirection, M):
    """The buffer as [rows][R*S] pixel indices (-1 = zero row): (rows < M, the padding rows of the last tile).
    Plans that keep two forms of the entries are decoded from both, which must agree."""
    L = icv.get_indirection_layout(p)
    T = p.R * p.S
    mr, tiles = L.tile_rows, L.tiles
    assert tiles == -(-M // mr) and icv.indirection_index(p, 0, 0) == 0
    if T > 1:
        assert icv.indirection_index(p, 0, 1) == mr
    raw = indirection.cpu().numpy().view(np.uint8)
    stride = _stride_bytes(p)
    n = tiles * T * mr
    forms = []
    if L.int32_entries_at >= 0:
        e = raw[L.int32_entries_at:L.int32_entries_at + 4 * n].view(np.int32).reshape(tiles, T, mr)
        assert np.all((e >= 0) | (e == np.iinfo(np.int32).min))
        assert np.all(e[e >= 0] % stride == 0)
        forms.append(np.where(e < 0, -1, e // stride))
    if L.entry_bytes == 2:
        rec, e = tile_records(p, indirection)
        off = rec[:, 0].astype(np.int64)[:, None, None] + e.astype(np.int64) * stride
        assert np.all(rec[:, 0] % stride == 0)
        forms.append(np.where(e == L.zero_code, -1, off // stride))
    else:
        assert L.entry_bytes == 4 and L.entries_at == L.int32_entries_at
    for f in forms[1:]:
        assert np.array_equal(forms[0], f)
    logical = forms[0].transpose(0, 2, 1).reshape(tiles * mr, T).astype(np.int32)
    return logical[:M], logical[M:]
