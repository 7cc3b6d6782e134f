"""Writes tests/golden/quantised_hashes.txt: SHA-256 of the oracle-quantised bytes and row scales of a few
synthetic matrices.  Calls the seeded generators (synth/) and the CPU oracle (oracle/) only; the test that reads
the file recomputes the same digests, so a change of the generator's draws, of their order, or of the oracle's
quantisation arithmetic shows up as a changed line.

    python tests/golden/write_quantised_hashes.py
"""
import hashlib
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle.quant as oq  # noqa: E402
import synth  # noqa: E402

# (rows, cols, layer, matrix index, rescale)
CASES = [(4096, 4096, 0, 0, False), (4096, 4096, 0, 0, True), (512, 11008, 0, 6, True), (640, 5120, 31, 3, False)]


def digests(rows, cols, layer, m, rescale):
    seed = synth.matrix_seed(layer, m)
    w = synth.gen_weight(rows, cols, seed)
    if rescale:
        w = oq.rescale(w, oq.channel_scale(synth.gen_act_absmax(cols, seed), 0.5))
    q, scale = oq.quantise_rows(w)
    q = oq.prune(q)
    return hashlib.sha256(q.tobytes()).hexdigest(), hashlib.sha256(scale.tobytes()).hexdigest()


def lines():
    out = ["# rows cols layer matrix rescale sha256(int8 bytes after pruning) sha256(fp32 row scales)",
           "# written by tests/golden/write_quantised_hashes.py from synth/ and oracle/quant.py alone"]
    for rows, cols, layer, m, rescale in CASES:
        hq, hs = digests(rows, cols, layer, m, rescale)
        out.append(f"{rows} {cols} {layer} {m} {int(rescale)} {hq} {hs}")
    return out


if __name__ == "__main__":
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "quantised_hashes.txt"), "w") as f:
        f.write("\n".join(lines()) + "\n")
    print("\n".join(lines()))
