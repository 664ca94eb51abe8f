"""Storage / operation / energy gains of CSR, CER and CSER over the dense representation, in the form of
the paper's Tables II, III, V and VI, for the synthetic stand-in matrices of this repository.

    python -m paper_1805_10692_amd.cost_tables [--markdown]

Everything is computed by the library's cost model (cer_cost_model / csr_cost_model / dense_cost_model:
elementary operations of ONE matrix-vector product as counted in Eq. (2), (4), (10), (12), storage bits
with per-array minimal index widths, energy priced with Table I); no GPU is needed.  Gains are
dense / format, as in the paper (> 1 means the format is better than dense).
"""
from __future__ import annotations

import argparse

from . import binding as B
from . import workloads as wl


def rows():
    cases = [
        ("alexnet_fc6 4096x9216 K=32 p0=0.85", lambda: wl.alexnet_fc6(L=1)),
        ("vgg_fc6 4096x25088 K=16 p0=0.95", lambda: wl.vgg_fc6(L=1)),
        ("conv3x3 512x4608 K=8 p0=0.6", lambda: wl.conv3x3(L=1)),
        ("conv3x3, most frequent value 0.25", lambda: wl.conv3x3(L=1, nonzero_dominant=True)),
        ("c1 256x512 K=16 p0=0.9", lambda: wl.config1()),
    ]
    for K in wl.SWEEP_K:
        for p0 in wl.SWEEP_P0:
            cases.append((f"sweep 2048x2048 K={K} p0={p0}", lambda K=K, p0=p0: wl.sweep_cell(K, p0, L=1)))
    for name, make in cases:
        w = make()
        dense = B.dense_cost_model(w.m, w.n)
        hc = B.cer_encode(w.W, w.codebook)
        hs = B.cser_encode(w.W, w.codebook)
        hr = B.csr_encode(w.W)
        st = B.cer_get_stats(hc)
        costs = {"csr": B.csr_cost_model(hr), "cer": B.cer_cost_model(hc), "cser": B.cer_cost_model(hs)}
        B.cer_free(hc)
        B.cer_free(hs)
        B.csr_free(hr)
        out = {"name": name, "H": st["H"], "p0": st["p0"], "k_bar": st["k_bar"], "k_tilde": st["k_tilde"],
               "dense_MB": dense["storage_bits"] / 8e6, "dense_Mops": dense["ops"] / 1e6,
               "dense_uJ": dense["energy_pj"] / 1e6}
        for f, c in costs.items():
            out[f"storage_{f}"] = dense["storage_bits"] / c["storage_bits"]
            out[f"ops_{f}"] = dense["ops"] / c["ops"]
            out[f"energy_{f}"] = dense["energy_pj"] / c["energy_pj"]
        yield out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--markdown", action="store_true")
    args = ap.parse_args()
    head = ["matrix", "H", "p0", "k_bar", "k_tilde", "dense MB", "storage CSR/CER/CSER", "dense Mops", "#ops CSR/CER/CSER",
            "dense uJ", "energy CSR/CER/CSER"]
    if args.markdown:
        print("| " + " | ".join(head) + " |")
        print("|" + "---|" * len(head))
    for r in rows():
        cells = [r["name"], f"{r['H']:.2f}", f"{r['p0']:.3f}", f"{r['k_bar']:.1f}", f"{r['k_tilde']:.1f}",
                 f"{r['dense_MB']:.2f}",
                 f"x{r['storage_csr']:.2f} / x{r['storage_cer']:.2f} / x{r['storage_cser']:.2f}",
                 f"{r['dense_Mops']:.2f}", f"x{r['ops_csr']:.2f} / x{r['ops_cer']:.2f} / x{r['ops_cser']:.2f}",
                 f"{r['dense_uJ']:.1f}", f"x{r['energy_csr']:.2f} / x{r['energy_cer']:.2f} / x{r['energy_cser']:.2f}"]
        print(("| " + " | ".join(cells) + " |") if args.markdown else "  ".join(cells), flush=True)
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
