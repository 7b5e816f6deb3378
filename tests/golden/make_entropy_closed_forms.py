"""Prints the closed-form entropy table in entropy_closed_forms.txt with 50-digit
decimal arithmetic (no oracle, no GPU code involved): uniform -> ln V; m logits at a
and V-m at 0 -> ln Z - a m e^a / Z with Z = m e^a + V - m."""
from decimal import Decimal, getcontext

getcontext().prec = 50


def uniform(V):
    return Decimal(V).ln()


def twolevel(V, m, a):
    a = Decimal(a)
    ea = a.exp()
    Z = m * ea + (V - m)
    return Z.ln() - a * m * ea / Z


if __name__ == "__main__":
    for V in (512, 4096, 2):
        print(f"uniform   {V:<5d} 0    0.0   {uniform(V):.32g}")
    for V, m, a in ((4, 1, "1.0"), (512, 1, "10.0"), (4096, 16, "3.0"), (4096, 1, "20.0")):
        print(f"twolevel  {V:<5d} {m:<4d} {a:<5s} {twolevel(V, m, a):.32g}")
