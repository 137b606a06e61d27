"""Writes tests/golden/tiny_case.json: a small paged decode-attention problem (inputs as raw bf16
bits) with the outputs the fp64 oracle computes for it.  Calls only `oracle/` and the seeded input
generator; run it from the repository root:  python tests/golden/make_tiny_case.py

The paper prints no worked numerical example of its attention step (it names the operation,
Sec. 2.1, and reports timings), so there is no printed value to store; this fixture freezes the
oracle's own answer on one case so that a later change to the oracle's arithmetic shows up as a
diff of this file."""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402
import workloads as W  # noqa: E402


def main():
    lens = np.asarray([0, 15, 17], dtype=np.int32)                 # tokens before the append
    wl = W.Workload(98, "golden", B=len(lens), Hq=2, Hkv=1, d=64, lengths="given", fixed_pool_pages=5)
    b = W.make_batch(wl, device="cpu", headroom_tokens=1, seed_offset=5, lens_before=lens)
    k, v = W.bits(b.k_cache).copy(), W.bits(b.v_cache).copy()
    oracle.kv_append(k, v, W.bits(b.k_new), W.bits(b.v_new), b.block_table, b.positions)
    out, lse, _ = oracle.decode_attention(W.bits(b.q), k, v, b.block_table, b.seq_lens, wl.scale)
    case = {
        "comment": "bf16 tensors as raw 16-bit patterns (the two caches as one hex string, 4 digits per element, "
                   "shape [pages][16][Hkv][d]); out/lse are the fp64 oracle's, printed with repr()",
        "num_pages": int(b.num_pages),
        "Hq": wl.Hq, "Hkv": wl.Hkv, "d": wl.d, "page_size": 16, "scale": wl.scale,
        "positions": b.positions.tolist(), "seq_lens": b.seq_lens.tolist(), "block_table": b.block_table.tolist(),
        "q": W.bits(b.q).tolist(), "k_new": W.bits(b.k_new).tolist(), "v_new": W.bits(b.v_new).tolist(),
        "k_cache_before": "".join("%04x" % x for x in W.bits(b.k_cache).reshape(-1)),
        "v_cache_before": "".join("%04x" % x for x in W.bits(b.v_cache).reshape(-1)),
        "out": [[[repr(float(x)) for x in row] for row in req] for req in out],
        "lse": [[repr(float(x)) for x in row] for row in lse],
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_case.json")
    with open(path, "w") as f:
        json.dump(case, f, separators=(",", ":"))
        f.write("\n")
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
