"""Exact-rational evaluation of the closed form of golden case A (adamw_hand_worked.txt,
[A_constant_gradient_two_steps]) with Python fractions: p_t = 0.875 p_(t-1) - 0.25 g / (|g| + 0.5),
m_t = (1 - b1^t) g, v_t = (1 - b2^t) g^2.  It evaluates the closed form written next to the case
and nothing else: no optimizer implementation, no oracle, no library.  It was used to do the
long-hand arithmetic of that case (the other cases were done on paper); run it to re-derive the
expected values printed in the fixture."""
from fractions import Fraction as F

g = [F(x) for x in (0, .5, -.5, 1.5, -1.5, 3.5, -3.5, 7.5, -7.5, .5, 1.5, 3.5, 7.5, -.5, -1.5, 0)]
p = [F(x) for x in (1, 1, 1, 1, 1, 1, 1, 1, 1, -2, -2, -2, -2, .5, .5, 1.00390625)]
u = [x / (abs(x) + F(1, 2)) for x in g]

if __name__ == "__main__":
    print("stored gradients (loss scale 4):", [float(4 * x) for x in g])
    for t, (one_minus_b1_t, one_minus_b2_t) in enumerate([(F(3, 4), F(1, 4)), (F(15, 16), F(7, 16))], 1):
        p = [F(7, 8) * a - F(1, 4) * b for a, b in zip(p, u)]
        print("t = %d" % t)
        print("  master    ", [float(x) for x in p])
        print("  exp_avg   ", [float(one_minus_b1_t * x) for x in g])
        print("  exp_avg_sq", [float(one_minus_b2_t * x * x) for x in g])
