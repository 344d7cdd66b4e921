"""Writes ramp_closed_form.json from the hand-derived formulas only (no oracle, no GPU).

Input x_i = i+1, i < N, K = 2^bits dividing N, nothing pruned or protected, m = N/K.  The
equal-frequency boundaries are t_j = j*m + 1, the bin means are k*m + (m+1)/2 and each bin's
squared error is m(m^2-1)/12 (variance of m consecutive integers times m), so SSE = K*m(m^2-1)/12.
The paper's System Overview equates 8 bins with 3 bits, i.e. K = 2^bits.
"""
import json
import os

cases = []
for N, bits in [(64, 3), (1024, 2), (4096, 8), (96, 5), (2, 1)]:
    K = 1 << bits
    m = N // K
    assert K * m == N
    cases.append(dict(N=N, bits=bits, boundaries=[float(j * m + 1) for j in range(1, K)],
                      codebook=[k * m + (m + 1) / 2 for k in range(K)],
                      sse=K * m * (m * m - 1) / 12))
with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "ramp_closed_form.json"), "w") as f:
    json.dump(dict(source="closed form; K = 2^bits per the paper's System Overview (8 bins = 3 bits)",
                   cases=cases), f, indent=1)
