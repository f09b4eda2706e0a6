"""Writes ffn_hand_d4.json: a hand-worked FFN block (d=4, f=2) whose result has a closed
form in p = Phi(1), the standard normal CDF at 1 (0.8413447460685429 in any table).

  x = [2,0,-2,0];  W1 = [[.5,0,0,0],[0,0,-.5,0]], b1 = 0  ->  h = [1,1]  ->  GELU(h) = [p,p]
  W2 = [[1,0],[0,1],[0,0],[1,1]], b2 = 0                   ->  [p,p,0,2p]
  z = x + that = [2+p, p, -2, 2p];  mean = p;  z - mean = [2, 0, -2-p, p]
  biased var = (4 + (2+p)^2 + p^2)/4;  eps = 0
  y = (z-mean)/sqrt(var) * g + beta,  g = [1,2,1,1], beta = [0,0,.5,0]

Uses neither the oracle nor the GPU library: it only evaluates the line above.
"""
import json
import math
import os

p = 0.8413447460685429
sd = math.sqrt((4.0 + (2.0 + p) ** 2 + p * p) / 4.0)
dev = [2.0, 0.0, -2.0 - p, p]
g = [1.0, 2.0, 1.0, 1.0]
beta = [0.0, 0.0, 0.5, 0.0]
y = [dev[i] / sd * g[i] + beta[i] for i in range(4)]
doc = {
    "cites": "Linear(a)=Wa+b and the residual block shape of Sec. 3.2.2; GELU(1)=Phi(1)",
    "x": [[2.0, 0.0, -2.0, 0.0]],
    "weights": {"w1": [[0.5, 0, 0, 0], [0, 0, -0.5, 0]], "b1": [0.0, 0.0],
                "w2": [[1.0, 0], [0, 1.0], [0, 0], [1.0, 1.0]], "b2": [0.0, 0.0, 0.0, 0.0],
                "ln_g": g, "ln_b": beta},
    "eps": 0.0,
    "y": [y],
}
with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "ffn_hand_d4.json"), "w") as fh:
    json.dump(doc, fh, indent=1)
