"""Pack / unpack by segment size: what the pack kernel makes of HBM.

Run as `python -m paper_2511_14124_amd.pack_probe`.  For every segment size from
64 B to 1 MiB one launch packs (then unpacks) 1 GiB of equal segments, with the
tensors at the slab's 16-byte phase and 4 bytes off it, and prints GB/s of read
plus written bytes.  Segments of under 512 B put more than 32 pieces into a
16 KiB tile and take the path with the workgroup-wide piece table.
"""

from __future__ import annotations

import numpy as np


def measure(torch, T, seg_bytes: int, total: int, shift: int, unpack: bool, reps: int = 4) -> float:
    dev = torch.device("cuda:0")
    n = total // seg_bytes
    nb = np.full(n, seg_bytes, dtype=np.uint64)
    off = np.arange(n, dtype=np.uint64) * np.uint64(seg_bytes)
    # tensors in reverse order of the slab, 256 bytes apart plus the shift
    stride = (seg_bytes + 255) // 256 * 256
    src = torch.empty(n * stride + 4096, dtype=torch.uint8, device=dev)
    slab = torch.empty(n * seg_bytes, dtype=torch.uint8, device=dev)
    src.random_(0, 255)
    src_off = (np.uint64(n - 1) - np.arange(n, dtype=np.uint64)) * np.uint64(stride) + np.uint64(shift)
    ptrs = torch.from_numpy((src_off + np.uint64(src.data_ptr())).astype(np.int64)).to(dev)
    nbt = torch.from_numpy(nb.astype(np.int64)).to(dev)
    offt = torch.from_numpy(off.astype(np.int64)).to(dev)
    st = torch.cuda.current_stream().cuda_stream
    tot = int(n) * seg_bytes
    index = torch.empty(T.pack_tiles(tot), dtype=torch.int32, device=dev)
    T.pack_index(offt.data_ptr(), n, tot, index.data_ptr(), st)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best = 1e30
    for _ in range(reps + 1):
        e0.record()
        (T.unpack if unpack else T.pack)(slab.data_ptr(), ptrs.data_ptr(), nbt.data_ptr(), offt.data_ptr(), n, tot, st,
                                         index.data_ptr())
        e1.record()
        e1.synchronize()
        best = min(best, e0.elapsed_time(e1))
    return 2.0 * tot / (best * 1e6)


def main():
    import torch
    from . import binding as T
    T.load_library()
    total = 1 << 30
    print("pack / unpack of 1 GiB of equal segments, GB/s of read + written bytes (HBM peak 8000)")
    print(f"{'segment':>10} {'pack':>8} {'unpack':>8} {'pack, 4 B off':>14} {'unpack, 4 B off':>16}")
    for seg in (64, 256, 1024, 4096, 16384, 65536, 262144, 1 << 20):
        row = [measure(torch, T, seg, total, shift, unpack) for shift in (0, 4) for unpack in (False, True)]
        print(f"{seg:>9}B {row[0]:>8.0f} {row[1]:>8.0f} {row[2]:>14.0f} {row[3]:>16.0f}", flush=True)


if __name__ == "__main__":
    main()
