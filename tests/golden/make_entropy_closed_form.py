"""Writes entropy_closed_form.txt: closed-form entropies of two-level logit
vectors, evaluated in 80-digit decimal arithmetic (standard library only).

H = ln(n e^a + V - n) - n a e^a / (n e^a + V - n)   [nats]
"""
import os
from decimal import Decimal, getcontext

getcontext().prec = 80

CASES = [  # (V, n, a)
    (50304, 1, "0"), (50304, 1, "5"), (50304, 1, "10"), (50304, 1, "20"), (50304, 1, "30"),
    (50304, 7, "12.5"), (50304, 1000, "3"), (50304, 50303, "4"),
    (8, 1, "2"), (8, 3, "1"), (2, 1, "0.5"),
]

here = os.path.dirname(os.path.abspath(__file__))
with open(os.path.join(here, "entropy_closed_form.txt"), "w") as f:
    f.write("# V n a H_nats lse   (n logits = a, V-n logits = 0; closed form, 80-digit decimal)\n")
    for V, n, a in CASES:
        a_d = Decimal(a)
        ea = a_d.exp()
        Z = n * ea + (V - n)
        H = Z.ln() - n * a_d * ea / Z
        f.write(f"{V} {n} {a} {H:.20e} {Z.ln():.20e}\n")
