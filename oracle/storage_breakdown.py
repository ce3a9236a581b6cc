"""How much each bf16 storage point of a bf16 deployment costs against the plain fp64 forward: oracle only, CPU.

TEST INFRASTRUCTURE (part of the oracle).  Runs the oracle's forward (Alg. 2 step 2) on one synthetic request of a
named model shape with no rounding, with every storage point rounded, with the set a deployment needs, and with each
point alone, and prints the worst-row differences of the logits.  The per-point figures quoted for the 1B and 8B
shapes come from

    python -m oracle.storage_breakdown llama1b 2048 9
    python -m oracle.storage_breakdown llama8b 1024 9      (needs ~40 GB of host memory and a few minutes)
"""
from __future__ import annotations

import sys

import numpy as np

from oracle import oracle
from paper_2601_00644_amd import synth      # seeded input generators only


def metrics(y: np.ndarray, ref: np.ndarray):
    rms = np.sqrt((ref * ref).mean(-1, keepdims=True))
    return (float((np.linalg.norm(y - ref, axis=-1) / np.linalg.norm(ref, axis=-1)).max()),
            float((np.abs(y - ref) / np.abs(ref).max(-1, keepdims=True)).max()),
            float((np.abs(y - ref) / np.maximum(np.abs(ref), rms)).max()))


def main(name: str, L: int, n: int, seed: int = 1):
    cfg = synth.MODELS[name]
    wn = synth.weights_to_numpy(cfg, synth.make_weights(cfg, seed))
    k, v = synth.make_kv_context(cfg, L, seed, 0)
    toks = np.random.default_rng(5).integers(0, cfg.vocab, n).astype(np.int32)

    def run(mask):
        kc, vc = oracle.new_cache(cfg, L + n)
        kc[:, :L], vc[:, :L] = synth.kv_to_f64(k), synth.kv_to_f64(v)
        return oracle.forward(cfg, wn, kc, vc, L, toks, stored=mask)

    ref = run(0)
    rows = [("all six points", 63), ("a + kv + o + act", oracle.ST_A | oracle.ST_KV | oracle.ST_O | oracle.ST_ACT)]
    rows += [("kv + o + act", oracle.ST_KV | oracle.ST_O | oracle.ST_ACT),
             ("a, o in fp16 + kv + act", oracle.ST_A16 | oracle.ST_O16 | oracle.ST_KV | oracle.ST_ACT),
             ("a, o in fp16 only", oracle.ST_A16 | oracle.ST_O16), ("kv only", oracle.ST_KV)]
    rows += [(f"only {nm}", bit) for nm, bit in oracle.ST_NAMES.items() if bit != oracle.ST_KV]
    print(f"{name}: context {L}, {n} rows, {cfg.n_layers} layers; difference of the logits from the fp64 forward")
    print(f"{'rounded to bf16':18s} {'worst row L2':>12s} {'elem / row max':>14s} {'elem / max(|ref|, rms)':>22s}")
    for tag, mask in rows:
        l2, row, elem = metrics(run(mask), ref)
        print(f"{tag:18s} {l2:12.4f} {row:14.4f} {elem:22.4f}", flush=True)


if __name__ == "__main__":
    main(sys.argv[1], int(sys.argv[2]), int(sys.argv[3]))
