"""What a bounded window would cost the vector-based LZ step (Section III-D, Table VI: windows of 32 to 255 vectors).

The library matches a row against the whole batch (first occurrence).  This script measures, on the synthetic
workload-3 tables and on the CPU, how many rows still find a match when only the last W rows may be referred to, and
what that does to the ratio: the rows that lose their match are coded like any other row.  It also prices the paper's
other arrangement, the LZ step as a compressor of its own (no entropy coder behind it), with a plain cost model.
Test infrastructure like the rest of this folder: it calls the oracle and the input generators only.

    python oracle/window_study.py [tables] [batch]
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import dlc_workloads as W  # noqa: E402
import oracle  # noqa: E402


def previous_occurrence_distance(sym_rows):
    """distance (in rows) from every row to the latest earlier row with the same symbols; 0 = none."""
    _, inv = np.unique(sym_rows, axis=0, return_inverse=True)
    inv = inv.reshape(-1)
    last = {}
    dist = np.zeros(inv.size, np.int64)
    for i, k in enumerate(inv.tolist()):
        if k in last:
            dist[i] = i - last[k]
        last[k] = i
    return dist


def main():
    T = int(sys.argv[1]) if len(sys.argv) > 1 else 8
    B = int(sys.argv[2]) if len(sys.argv) > 2 else 8192
    w = W.workload3(T=T, B=B, D=128)
    x = np.asarray(w.payload)
    lo, hi = x.min(axis=(1, 2)), x.max(axis=(1, 2))
    ebs = (0.03 * (hi - lo)).astype(np.float32)   # one bound per table, range-relative like the benchmark
    plain = oracle.compress(x, ebs)
    whole = oracle.compress(x, ebs, row_match=True)
    raw = x.nbytes
    print(f"{T} tables x {B} rows x 128, bounds 0.03 of the range")
    print(f"entropy coder alone: ratio {raw / plain.data.size:.2f};  whole-batch window + entropy coder (the library): ratio {raw / whole.data.size:.2f}")
    dist = []
    for t in range(T):
        sym, _ = oracle.quantize(x[t:t + 1], float(ebs[t]))
        dist.append(previous_occurrence_distance(sym[0]))
    dist = np.stack(dist)
    matched_whole = float((dist > 0).mean())
    # bytes of a coded row and of a reference under the entropy coder, from the two containers above
    ref_bytes = 4.0
    coded_rows_whole = (1.0 - matched_whole) * T * B
    row_bytes = (whole.data.size - ref_bytes * T * B) / coded_rows_whole
    print(f"rows with an earlier equal row: {matched_whole:.3f};  a coded row costs {row_bytes:.1f} bytes, a reference {ref_bytes:.0f}")
    print("window   rows matched   ratio with entropy coder (model)   ratio as LZ alone, 16-bit literals (model)")
    for win in (32, 64, 128, 255, B):
        m = float(((dist > 0) & (dist <= win)).mean())
        rb = 1.0 if win <= 255 else 4.0           # a reference fits a byte when the window does
        with_huffman = raw / (T * B * ((1.0 - m) * row_bytes + rb))
        alone = raw / (T * B * ((1.0 - m) * 128 * 2.0 + rb))
        print(f"{win:6d}   {m:12.3f}   {with_huffman:32.2f}   {alone:40.2f}")


if __name__ == "__main__":
    main()
