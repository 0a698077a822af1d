"""Writes closed_forms.json: textbook values of the scalar functions and the small worked
examples used to pin the oracle.  Uses Python's ``math`` module only (IEEE double libm);
it calls neither the oracle nor the GPU library.

The paper prints no numeric worked example for this path (its figures carry all numbers),
so these are mathematical closed forms: sigma(x) = 1/(1+e^-x), tanh, log-sum-exp.
Run:  python tests/golden/make_closed_forms.py
"""
import json
import math
import os


def sigma(x):
    return 1.0 / (1.0 + math.exp(-x))


def main():
    out = {"_source": "closed forms evaluated with Python math (double); no oracle involved"}
    out["sigmoid"] = {str(x): sigma(x) for x in (0.0, 1.0, -1.0, 2.0)}
    out["tanh"] = {str(x): math.tanh(x) for x in (0.5, 1.5, 2.0)}
    # workload 1 on X=[[0,1],[-1,2]], b=[[0,1]], a=0.5 : tanh(a*X+b)
    out["c1_tiny"] = [[math.tanh(0.5 * 0 + 0), math.tanh(0.5 * 1 + 1)],
                      [math.tanh(0.5 * -1 + 0), math.tanh(0.5 * 2 + 1)]]
    # workload 2: (i,f,o,g) pre-activations and c_prev -> (c, h)
    def cell(zi, zf, zo, zg, cp):
        c = sigma(zf) * cp + sigma(zi) * math.tanh(zg)
        return c, sigma(zo) * math.tanh(c)
    out["c2_tiny"] = {"zeros_cprev1": cell(0, 0, 0, 0, 1.0),
                      "i1_f-1_o2_g0.5_cprev0.25": cell(1, -1, 2, 0.5, 0.25)}
    # workload 3 on the row [1,2,3]
    m = 3.0
    S = math.exp(1 - m) + math.exp(2 - m) + math.exp(3 - m)
    out["c3_tiny"] = {"m": m, "S": S, "lsm_t2": 3 - m - math.log(S), "loss_t2": -(3 - m - math.log(S)),
                      "loss_t0": -(1 - m - math.log(S)), "argmax": 2}
    out["ln_10000"] = math.log(10000.0)
    # E[max(0, s*z+t)] for z ~ N(0,1): t*Phi(t/s) + s*phi(t/s)
    def relu_mean(s, t):
        Phi = 0.5 * (1 + math.erf(t / s / math.sqrt(2)))
        phi = math.exp(-0.5 * (t / s) ** 2) / math.sqrt(2 * math.pi)
        return t * Phi + s * phi
    out["relu_mean"] = {"s1_t0": relu_mean(1, 0), "s1.5_t0.5": relu_mean(1.5, 0.5),
                        "s0.5_t-0.5": relu_mean(0.5, -0.5)}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "closed_forms.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
        f.write("\n")


if __name__ == "__main__":
    main()
