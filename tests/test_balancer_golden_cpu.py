"""Algorithm 1 (appendix A) pinned by candidate tables that were worked by hand
(tests/golden/balancer_alg1_cases.txt: every number there comes from the algorithm's
statements, none from a program).  This file holds no formula of the method: it only
compares.  The oracle's table and choice must equal the file; the C ABI's choice and
the two times it reports for it must equal the file too; and two planted mistakes in a
copy of the oracle (the iteration count rounded down, the last iteration's context
rounded up) must be caught by the same comparison."""
import os
import re

import pytest

from oracle import cronus_oracle as orc
from paper_2509_17357_amd import binding as B

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "balancer_alg1_cases.txt")


def load_cases():
    cases, cur = [], None
    for raw in open(GOLDEN):
        line = raw.split("#", 1)[0].strip()
        if not line:
            continue
        word, _, rest = line.partition(" ")
        if word == "case":
            cur = {"name": rest.strip(), "cand": []}
            cases.append(cur)
        elif word == "in":
            cur["in"] = {k: float(v) if "." in v else int(v) for k, v in re.findall(r"(\w+)=(\S+)", rest)}
        elif word == "cand":
            f = rest.split()
            cur["cand"].append((int(f[0]), int(f[1]), int(f[2]), float(f[3]), float(f[4])))
        elif word == "pick":
            cur["pick"] = int(rest)
        else:
            raise ValueError(line)
    assert len(cases) >= 8 and all("in" in c and "pick" in c for c in cases)
    return cases


CASES = load_cases()


def distinct(rows):
    out = []
    for r in rows:
        if not out or out[-1][0] != r[0]:
            out.append(r)
    return out


def check_against(mod, case):
    """Compare one case with the functions of `mod` (the oracle, or a mutated copy)."""
    a = case["in"]
    model = dict(k_p=a["k_p"], b_p=a["b_p"], k_ctxp=a["k_ctxp"], k_ctxd=a["k_ctxd"], b_c=a["b_c"])
    if case["cand"]:
        rows = mod.balancer_table(a["l_in"], a["n_d"], a["l_ctxd"], batch_tokens=a["B"], n_candidates=a["n_cand"],
                                  **model)
        assert len(rows) == a["n_cand"]
        assert distinct(rows) == case["cand"], case["name"]
    got = mod.balancer_split(a["l_in"], a["n_d"], a["l_ctxd"], a["n_free"], n_size=a["n_size"], batch_tokens=a["B"],
                             n_candidates=a["n_cand"], **model)
    assert got == case["pick"], case["name"]


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
def test_oracle_reproduces_the_hand_worked_tables(case):
    check_against(orc, case)


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
def test_c_abi_reproduces_the_hand_worked_choice_and_times(case):
    a = case["in"]
    l_p, tp, tc = B.cronus_balancer_split(a["l_in"], a["n_d"], a["l_ctxd"], a["n_free"], a["k_p"], a["b_p"],
                                          a["k_ctxp"], a["k_ctxd"], a["b_c"], n_size=a["n_size"],
                                          batch_tokens=a["B"], n_candidates=a["n_cand"], with_times=True)
    assert l_p == case["pick"]
    if case["cand"]:
        row = next(r for r in case["cand"] if r[0] == l_p)
        assert (tp, tc) == (row[3], row[4])
    else:
        assert tc == 0.0


MUTANTS = {
    "iteration count rounded down": ("n_iter = -(-l_c // n_p)", "n_iter = l_c // n_p"),
    "iteration count one too many": ("n_iter = -(-l_c // n_p)", "n_iter = l_c // n_p + 1"),
    "whole iterations rounded up": ("l_last = l_p + (l_c // n_p) * n_p", "l_last = l_p + (-(-l_c // n_p)) * n_p"),
    "last context one chunk short": ("l_last = l_p + (l_c // n_p) * n_p", "l_last = l_p + (l_c // n_p - 1) * n_p"),
    "mean of first and last context": ("(l_in + l_last) / 2.0", "(l_p + l_last) / 2.0"),
    "candidates rounded down": ("l_p = -(-j * l_in // n_candidates)", "l_p = max(1, j * l_in // n_candidates)"),
    "last minimum kept": ("gap < best_gap", "gap <= best_gap"),
    "capacity in tokens": ("n_free < -(-l_in // n_size)", "n_free < l_in // n_size"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistakes_in_a_copy_of_the_oracle_are_caught(name):
    """The pin has teeth: each single-statement mistake, planted in a copy of the oracle's
    source (on the CPU), fails the comparison with the hand-worked file."""
    old, new = MUTANTS[name]
    src = open(orc.__file__).read()
    assert src.count(old) == 1, "the oracle's statement moved: update the mutant"
    ns = {"__name__": "oracle_mutant"}
    exec(compile(src.replace(old, new), "oracle_mutant.py", "exec"), ns)

    class Mod:
        balancer_table = staticmethod(ns["balancer_table"])
        balancer_split = staticmethod(ns["balancer_split"])

    failed = 0
    for case in CASES:
        try:
            check_against(Mod, case)
        except (AssertionError, ZeroDivisionError):
            failed += 1
    assert failed > 0, name


def test_no_prefill_token_left_is_an_error_on_both_sides():
    with pytest.raises(ValueError):
        orc.balancer_split(1000, 512, 5000, 100, 1e-4, 0.0, 1e-6, 1e-7, 0.01)
    with pytest.raises(ValueError):
        orc.balancer_table(1000, 600, 5000, 1e-4, 0.0, 1e-6, 1e-7, 0.01)
    assert B.cronus_balancer_split(1000, 512, 5000, 100, 1e-4, 0.0, 1e-6, 1e-7, 0.01, check=False) == \
        B.CRONUS_ERR_INVALID_ARG
