"""Writes backward_scalar_example.json: the hand derivation of the scalar backward example, evaluated term by term.
Calls nothing but Python arithmetic (no oracle, no GPU library): the expressions below ARE the hand-worked example."""
import json
import os

alpha, w, beta, theta = 25.0, 0.75, 0.5, 1.0
x = [1, 1, 0]                                   # input spike train
v = [0.75, 1.125, 0.0625]                       # membrane before the reset: .75; .5*.75+.75 (spike -> .125); .5*.125
spikes = [0, 1, 0]
g_out = [1.0, -2.0, 0.5]                        # dL/ds_n, chosen freely
sg = [1.0 / (1.0 + alpha * abs(vn - theta)) ** 2 for vn in v]     # 1/7.25^2, 1/4.125^2, 1/24.4375^2
res = {}
for key, detached in (("not_detached", False), ("detached", True)):
    c, gv = 0.0, [0.0, 0.0, 0.0]
    for n in (2, 1, 0):
        gv[n] = g_out[n] * sg[n] + c * (1.0 if detached else 1.0 - theta * sg[n])
        c = beta * gv[n]
    res[key] = {"dY": gv, "dW_centre": sum(gv[n] * x[n] for n in range(3)), "g_in": [gv[n] * w for n in range(3)]}
doc = {"_citation": "Hand-worked backward pass of the per-step layer (1x1 image, centre tap 0.75, beta 0.5, theta 1, input "
                    "[1, 1, 0]) with the fast-sigmoid surrogate ds/dV = 1/(1 + alpha |V - theta|)^2, alpha = 25 (Sec. 5.1 "
                    "'Training' names surrogate and alpha; the formula is the published one of that name). Forward: V = 0.75, "
                    "1.125 (spike, reset to 0.125), 0.0625. Surrogate slopes: 1/7.25^2, 1/4.125^2, 1/24.4375^2. Backwards "
                    "from the last step with c = dL/dV' (0 after the last step): dL/dV_n = g_n sg_n + c (1 - theta sg_n) "
                    "[detached reset: + c], c <- beta dL/dV_n. dY_n = dL/dV_n (one step per group); dW_centre = sum_n dY_n "
                    "x_n; dL/dx_n = 0.75 dY_n. Written by make_backward_scalar_example.py, which evaluates exactly these "
                    "expressions.",
       "beta": beta, "theta": theta, "centre_tap": w, "alpha": alpha, "input": x, "spikes": spikes, "v_pre": v,
       "g_out": g_out, "surrogate_slopes": sg, **res}
json.dump(doc, open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "backward_scalar_example.json"), "w"), indent=1)
