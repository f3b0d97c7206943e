"""Plain CPU statement of the pack / unpack and batched copy / exchange
operations of the migration path.

TEST INFRASTRUCTURE ONLY: shares no code with the HIP library and is imported
by tests alone.

These operations have a plain definition (they are not in the paper, which
moves every tensor by itself; they are the batched movers this library puts
under Alg. 3's "async copy" lines), so the oracle is that definition written
out with one slice assignment per segment:

* pack:     slab[off_i : off_i + n_i] = tensor_i            for every segment i
* unpack:   tensor_i = slab[off_i : off_i + n_i]
* copy:     dst_i[:] = src_i
* exchange: per unit, both sources are read in full before either destination
            is written, so a unit may swap two buffers in place.

Pins: tests/test_oracle_pins.py checks pack against numpy.concatenate for
gap-free layouts, unpack(pack(x)) == x, and exchange on overlapping buffers
against a hand-written swap.
"""

from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np


def pack(tensors: Sequence[np.ndarray], slab_off: Sequence[int], slab: np.ndarray) -> np.ndarray:
    """Gather: tensor i lands at slab_off[i].  Bytes of the slab that no
    segment covers keep their value.  Returns the slab."""
    for t, o in zip(tensors, slab_off):
        n = int(t.shape[0])
        slab[int(o):int(o) + n] = t
    return slab


def unpack(slab: np.ndarray, sizes: Sequence[int], slab_off: Sequence[int]) -> List[np.ndarray]:
    """Scatter: the reverse of pack."""
    return [slab[int(o):int(o) + int(n)].copy() for n, o in zip(sizes, slab_off)]


def exchange(mem: np.ndarray, units: Sequence[Tuple[int, int, int, int, int]]) -> np.ndarray:
    """Units (out_src, out_dst, in_src, in_dst, n) over one flat byte array
    `mem`; a negative out_src or in_src leaves that half out.  Within a unit
    both reads happen before both writes; units are applied in order (a batch
    must not make one unit's source another unit's destination)."""
    for (os_, od, is_, id_, n) in units:
        o = mem[os_:os_ + n].copy() if os_ >= 0 else None
        i = mem[is_:is_ + n].copy() if is_ >= 0 else None
        if o is not None:
            mem[od:od + n] = o
        if i is not None:
            mem[id_:id_ + n] = i
    return mem
