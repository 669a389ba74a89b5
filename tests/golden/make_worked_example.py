"""Writes worked_example.txt: the 2-token, 3-expert layer of test_worked_example_by_hand, evaluated
by scalar arithmetic only (no oracle, no kernels).  Run: python tests/golden/make_worked_example.py"""
import math
import os

sig = lambda z: 1.0 / (1.0 + math.exp(-z))
silu = lambda z: z * sig(z)

# token 0: x = (1, 0)  -> logits = Wg row 0 = (1, 0, -1)            -> experts (0, 1)
# token 1: x = (0, 2)  -> logits = 2 * Wg row 1 = (1, .5, .5)       -> experts (0, 1), tie 1 vs 2 -> 1
w00 = sig(1.0 - 0.0)          # softmax over two logits = logistic of their difference
w10 = sig(1.0 - 0.5)
# expert 0: W1 = [[1,-1],[2,0]], W3 = [[.5,1],[1,1]], W2 = identity
y00 = (silu(1.0) * 0.5, silu(-1.0) * 1.0)        # x=(1,0): g=(1,-1), u=(.5,1)
y10 = (silu(4.0) * 2.0, silu(0.0) * 2.0)         # x=(0,2): g=(4,0),  u=(2,2)
# expert 1: W1 = [[0,1],[1,0]], W3 = [[1,1],[.5,-1]], W2 = [[0,1],[2,0]]  (y = (2*h1, h0))
h01 = (silu(0.0) * 1.0, silu(1.0) * 1.0)         # x=(1,0): g=(0,1), u=(1,1)
y01 = (2.0 * h01[1], h01[0])
h11 = (silu(2.0) * 1.0, silu(0.0) * -2.0)        # x=(0,2): g=(2,0), u=(1,-2)
y11 = (2.0 * h11[1], h11[0])
out0 = [w00 * y00[c] + (1 - w00) * y01[c] for c in range(2)]
out1 = [w10 * y10[c] + (1 - w10) * y11[c] for c in range(2)]
path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "worked_example.txt")
with open(path, "w") as fh:
    fh.write("# Hand-derived MoE layer: d=2, E=3, k=2, f=2 (the paper prints no worked example of the layer;\n"
             "# this one is derived by scalar arithmetic in make_worked_example.py, see the comments there).\n"
             "# rows: out[token 0], out[token 1]\n")
    fh.write("%.15e %.15e\n%.15e %.15e\n" % (out0[0], out0[1], out1[0], out1[1]))
print(open(path).read())
