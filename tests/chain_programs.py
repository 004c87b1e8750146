"""Seeded generator of random postfix chain programs (text only; none of the method's arithmetic)
shared by the CPU pin of the interpreter and the GPU parity test of run-time compiled chains."""
import random


def random_program(rng):
    """A random postfix chain over every primitive, built from two kinds of sub-expression so
    that values stay finite and well-conditioned for |x| <= 6: B (bounded) and L (grows at
    most linearly with x).  Only the program TEXT is made here; its meaning comes from the
    interpreter on one side and the library's compiler on the other."""
    consts = ["0.5", "1", "2", "-1.5", "0.25", "3"]

    def B(d):
        r = rng.randrange(9 if d > 0 else 4)
        if r == 0:
            return f"{L(d - 1)} tanh"
        if r == 1:
            return f"{L(d - 1)} sigmoid"
        if r == 2:
            return f"{L(d - 1)} erf"
        if r == 3:
            return rng.choice(consts)
        if r == 4:
            return f"{L(d - 1)} abs neg exp"
        if r == 5:
            return f"{L(d - 1)} {L(d - 1)} abs 1 + /"
        if r == 6:
            return f"{B(d - 1)} {B(d - 1)} {rng.choice(['+', '-', '*', 'min', 'max'])}"
        if r == 7:
            return f"{B(d - 1)} tanh exp"
        return f"{L(d - 1)} softplus tanh"            # the fused pair

    def L(d):
        if d <= 0:
            return "x"
        r = rng.randrange(10)
        if r == 0:
            return "x"
        if r == 1:
            return f"{L(d - 1)} {B(d - 1)} {rng.choice(['+', '-'])}"
        if r == 2:
            return f"{B(d - 1)} {L(d - 1)} *"
        if r == 3:
            return f"{L(d - 1)} softplus"
        if r == 4:
            return f"{L(d - 1)} {rng.choice(['relu', 'abs', 'neg'])}"
        if r == 5:
            return f"{L(d - 1)} abs 1 + log"
        if r == 6:
            return f"{L(d - 1)} abs 0.5 + sqrt"
        if r == 7:
            return f"{L(d - 1)} {L(d - 1)} {rng.choice(['+', '-', 'min', 'max'])}"
        if r == 8:
            return f"{L(d - 1)} {rng.choice(consts)} /"
        return f"{rng.choice(consts)} {L(d - 1)} *"

    return L(3) if rng.random() < 0.5 else B(3)


def random_programs(count, seed=20220922, max_tokens=60):
    rng = random.Random(seed)
    programs = []
    while len(programs) < count:
        p = random_program(rng)
        if "x" in p.split() and len(p.split()) <= max_tokens and p not in programs:
            programs.append(p)
    return programs
