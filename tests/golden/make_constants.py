"""Writes closed_form_constants.txt: values of the logistic function and of
softplus at the score gaps the two-key oracle pins use.  Computed with the
standard library's arbitrary-precision decimal arithmetic (50 digits), so they
depend on neither the oracle nor libm.  The paper prints no numeric example for
Flash Decode; these are the mathematics of a two-key softmax:
weight = 1/(1+e^-x), lse - s2 = ln(1+e^x) for score gap x = s1 - s2.
"""
import os
from decimal import Decimal, getcontext

getcontext().prec = 50


def sigmoid(x: Decimal) -> Decimal:
    return 1 / (1 + (-x).exp())


def softplus(x: Decimal) -> Decimal:
    return (1 + x.exp()).ln()


rows = [("1", Decimal(1)), ("2", Decimal(2)), ("sqrt2", Decimal(2).sqrt())]
here = os.path.dirname(os.path.abspath(__file__))
with open(os.path.join(here, "closed_form_constants.txt"), "w") as fh:
    fh.write("# two-key softmax closed forms (score gap x): weight sigmoid(x), lse gap softplus(x)\n")
    fh.write("# written by make_constants.py with 50-digit decimal arithmetic; 20 digits kept\n")
    for name, x in rows:
        fh.write(f"sigmoid_{name} = {sigmoid(x):.20f}\n")
        fh.write(f"softplus_{name} = {softplus(x):.20f}\n")
