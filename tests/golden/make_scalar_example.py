"""Writes scalar_example.txt: the attention-softmax path for H=1, S=2, T=1, V=2.

At this size every step of section 3.2 (Eq. 1-6) collapses to a scalar
textbook function, evaluated here with Python's math module only (no numpy, no
oracle, no GPU code): the two-way attention softmax is the logistic sigmoid of
the score difference, the output softmax loss is softplus(l0 - l1).
Run from the repository root:  python tests/golden/make_scalar_example.py
"""
import math
import os

h_dec, h_enc1, h_enc2 = 0.5, 0.8, -0.4
W_a = 1.5
W_c_c, W_c_h = 0.7, -0.3          # columns acting on the context c and on h_t
W_out0, W_out1 = 0.9, -0.6
b_out0, b_out1 = 0.1, 0.2
# target word is id 1

sig = lambda x: 1.0 / (1.0 + math.exp(-x))
alpha1 = sig(h_dec * W_a * (h_enc1 - h_enc2))                    # Eq. 1-2
c = alpha1 * h_enc1 + (1 - alpha1) * h_enc2                      # Eq. 3
h_tilde = math.tanh(W_c_c * c + W_c_h * h_dec)                   # Eq. 4
l0, l1 = W_out0 * h_tilde + b_out0, W_out1 * h_tilde + b_out1    # Eq. 5
loss = math.log1p(math.exp(l0 - l1))                             # -log P(y=1), Eq. 6
p0 = sig(l0 - l1)
dz = p0 * (W_out0 - W_out1) * (1 - h_tilde ** 2)
dc = dz * W_c_c
dW_a = dc * alpha1 * (1 - alpha1) * (h_enc1 - h_enc2) ** 2 * h_dec

out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "scalar_example.txt")
with open(out, "w") as fh:
    fh.write("# Scalar worked example of section 3.2, Eq. 1-6 (H=1, S=2, T=1, V=2, target id 1).\n")
    fh.write("# Written by make_scalar_example.py from closed forms (sigmoid, tanh, softplus).\n")
    for k, v in [("h_dec", h_dec), ("h_enc1", h_enc1), ("h_enc2", h_enc2), ("W_a", W_a),
                 ("W_c_c", W_c_c), ("W_c_h", W_c_h), ("W_out0", W_out0), ("W_out1", W_out1),
                 ("b_out0", b_out0), ("b_out1", b_out1)]:
        fh.write(f"{k} = {v!r}\n")
    fh.write("# expected\n")
    for k, v in [("alpha1", alpha1), ("h_tilde", h_tilde), ("loss", loss), ("db_out0", p0), ("dW_a", dW_a)]:
        fh.write(f"{k} = {v:.12f}\n")
