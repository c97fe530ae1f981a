"""Fidelity of token-wise FP4 quantization of activations under the two readings of the clamp's
scope (Sec. 3.2, Table 1's three metrics): cosine similarity, MSE and SNR between an activation
tensor and its reconstruction, without clamp, with clamp, and with clamp plus the residual, for
thresholds taken per tensor and per token.  Synthetic activations only (the recipes of the GPU
workloads); the paper's own numbers need its training runs.

Test infrastructure like the rest of this directory.  Usage:  python -m oracle.fidelity_table
Prints a markdown table; the design notes quote it."""
import numpy as np

from oracle import fp4_oracle as o
from paper_2501_17116_amd import synth


def rows(cfg_name: str, tokens: int = 2048):
    cfg = synth.CONFIGS[cfg_name]
    layer = cfg.layers[0]
    A = synth.make_activation(cfg, tokens, layer.K, 0).numpy()
    out = [("no clamp", "-", "-") + o.fidelity(A, o.dequantized_activation(A, None, False))]
    for alpha in (0.999, 0.99, 0.97):
        for scope in ("tensor", "token"):
            for comp in (False, True):
                rec = o.dequantized_activation(A, alpha, comp, scope=scope)
                out.append(("clamp + residual" if comp else "clamp", "%g" % alpha, scope) + o.fidelity(A, rec))
    return layer, out


def main():
    for name in ("c3", "c4"):
        layer, table = rows(name)
        print("\n%s activations, 2048 tokens x %d channels\n" % (name, layer.K))
        print("| treatment | alpha | thresholds | SIM | MSE | SNR (dB) |")
        print("|---|---|---|---:|---:|---:|")
        for what, alpha, scope, sim, mse, snr in table:
            print("| %s | %s | %s | %.4f | %.4g | %.2f |" % (what, alpha, scope, sim, mse, snr))


if __name__ == "__main__":
    main()
