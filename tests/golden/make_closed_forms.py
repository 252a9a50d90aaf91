"""Writes closed_forms.txt: values fixed by the paper's formulas alone.

Nothing here calls the oracle or the GPU library.  Each value is a closed form
that algebra gives for a special case of the paper's equations, evaluated in
60-digit arithmetic and printed to 17 significant digits.

* vstar_binary G k beta: Eq. 2 (Sec. 3.1) with binary rewards, k of the G
  rollouts rewarded 1:  V* = beta * ln(1 + (k/G) (e^{1/beta} - 1)).
* loss_onpolicy G k beta: Eq. 3 (Sec. 3.1) with pi = pi_vllm, one prompt with
  k of G rewarded 1:  L = k (1 - V*)^2 + (G - k) V*^2.
* ln_vocab V: log-prob of any token under a uniform soft-max, -ln V.
"""
import os

import mpmath

mpmath.mp.dps = 60


def vstar_binary(G, k, beta):
    beta = mpmath.mpf(beta)
    return beta * mpmath.log1p(mpmath.mpf(k) / G * mpmath.expm1(1 / beta))


def main():
    lines = ["# kind args... value   (see make_closed_forms.py for the formulas and citations)"]
    for G, k, beta in [(8, 2, "1"), (8, 2, "0.5"), (8, 1, "2"), (4, 2, "1"), (16, 5, "1"),
                       (8, 3, "0.001"), (8, 3, "1000"), (8, 0, "1"), (8, 8, "0.5"), (4, 1, "1")]:
        v = vstar_binary(G, k, beta)
        lines.append(f"vstar_binary {G} {k} {beta} {mpmath.nstr(v, 17)}")
        L = k * (1 - v) ** 2 + (G - k) * v ** 2
        lines.append(f"loss_onpolicy {G} {k} {beta} {mpmath.nstr(L, 17)}")
    for V in (2, 1024, 151936):
        lines.append(f"ln_vocab {V} {mpmath.nstr(mpmath.log(V), 17)}")
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "closed_forms.txt")
    with open(out, "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
