"""Schedule search (Sec. 3: smallest l with every intermediate of order <= l): the result must pass
the legality check of Sec. 3.2, and l must equal the minimum found by brute force over every
pair of loop orders (the check itself is pinned against the paper's examples elsewhere)."""
import itertools
import re

import pytest

import paper_2401_04836_amd as cst
from paper_2401_04836_amd import schedules as S


def _norm(t):
    return re.sub(r"\s+", "", t)


def _brute_min_l(stmts, operands):
    """stmts: list of (lhs_ref, a_ref, b_ref, index set).  Every combination of loop orders through
    conststn_schedule_check; returns the smallest achievable maximum order of an intermediate."""
    best = None
    for perms in itertools.product(*[itertools.permutations(sorted(ix)) for _, _, _, ix in stmts]):
        text = " ; ".join("%s = %s * %s | %s" % (o, a, b, ",".join(p)) for (o, a, b, _), p in zip(stmts, perms))
        try:
            _, red = cst.schedule_check(text, operands)
        except cst.ConststnError:
            continue                                   # illegal for a CSF level order
        worst = max(red[:-1])
        best = worst if best is None else min(best, worst)
    return best


def test_tuned_schedules_are_what_the_search_returns():
    X = ("X", ("csf", (5, 6, 7)))
    text, l, modes = cst.schedule_search("T[i,j,s] = X[i,j,k] * U3[k,s] ; Y[i,r,s] = T[i,j,s] * U2[j,r]",
                                         [X, ("U3", (7, 3)), ("U2", (6, 2))], flags=cst.SEARCH_KEEP_LAYOUT)
    assert l == 1 and _norm(text) == _norm(S.TTMC3) and modes[0] == [0, 1, 2]
    text, l, _ = cst.schedule_search("T[i,j,r] = X[i,j,k] * C[k,r] ; M[i,r] = T[i,j,r] * B[j,r]",
                                     [X, ("C", (7, 3)), ("B", (6, 3))], flags=cst.SEARCH_KEEP_LAYOUT)
    assert l == 1 and _norm(text) == _norm(S.MTTKRP3)
    # statements given consumer first: the search orders them
    text2, l2, _ = cst.schedule_search("M[i,r] = T[i,j,r] * B[j,r] ; T[i,j,r] = X[i,j,k] * C[k,r]",
                                       [X, ("C", (7, 3)), ("B", (6, 3))], flags=cst.SEARCH_KEEP_LAYOUT)
    assert l2 == 1 and _norm(text2) == _norm(S.MTTKRP3)


@pytest.mark.parametrize("xref,dims", [("X[i,j,k]", (5, 6, 7)), ("X[k,j,i]", (7, 6, 5)), ("X[j,k,i]", (6, 7, 5)),
                                       ("X[k,i,j]", (7, 5, 6))])
def test_minimal_l_against_brute_force_with_a_fixed_layout(xref, dims):
    ops = [("X", ("csf", dims)), ("U3", (7, 3)), ("U2", (6, 2))]
    tree = "T[i,j,s] = %s * U3[k,s] ; Y[i,r,s] = T[i,j,s] * U2[j,r]" % xref
    text, l, _ = cst.schedule_search(tree, ops, flags=cst.SEARCH_KEEP_LAYOUT)
    _, red = cst.schedule_check(text, ops)
    assert max(red[:-1]) <= l
    want = _brute_min_l([("T[i,j,s]", xref, "U3[k,s]", "ijks"), ("Y[i,r,s]", "T[i,j,s]", "U2[j,r]", "ijrs")], ops)
    assert l == max(want, 1)                             # the question is first asked for l = 1 (Sec. 3)


def test_free_layout_chooses_the_level_order():
    # X given by modes (k, j, i): the search is free to store it i > j > k
    ops = [("X", ("csf", (7, 6, 5))), ("U3", (7, 3)), ("U2", (6, 2))]
    text, l, modes = cst.schedule_search("T[i,j,s] = X[k,j,i] * U3[k,s] ; Y[i,r,s] = T[i,j,s] * U2[j,r]", ops)
    assert l == 1 and modes[0] == [2, 1, 0] and "X[i,j,k]" in text
    # the schedule holds for X described in its new level order
    _, red = cst.schedule_check(text, [("X", ("csf", (5, 6, 7))), ("U3", (7, 3)), ("U2", (6, 2))])
    assert red[0] == 1


def test_running_example_of_the_paper():
    # Sec. 3.1: X = A x B, Y = X x C, R = Y x D, all four inputs sparse, layouts free
    tree = ("X[i,j,q,r] = A[i,p,q] * B[j,p,r] ; Y[i,j,k,r] = X[i,j,q,r] * C[k,q,r] ; "
            "R[i,j,k] = Y[i,j,k,r] * D[j,k,r]")
    dims = {"i": 4, "j": 7, "k": 9, "p": 5, "q": 6, "r": 8}
    ops = [("A", ("csf", (4, 5, 6))), ("B", ("csf", (7, 5, 8))), ("C", ("csf", (9, 6, 8))), ("D", ("csf", (7, 9, 8)))]
    text, l, modes = cst.schedule_search(tree, ops)
    assert l == 1
    # check it as a schedule over the layouts chosen
    refs = dict(re.findall(r"([ABCD])\[([a-z,]+)\]", text))
    chosen = [(n, ("csf", tuple(dims[c] for c in refs[n].split(",")))) for n in "ABCD"]
    lowered, red = cst.schedule_check(text, chosen)
    assert red[:2] == [1, 1]
    for o, n in enumerate("ABCD"):                      # level_modes maps levels back to the reference in the tree
        given = dict(re.findall(r"([ABCD])\[([a-z,]+)\]", tree))[n].split(",")
        assert [given[d] for d in modes[o]] == refs[n].split(",")
    # the fused structure the paper prints (intermediates of order 2) is one of the legal schedules too
    printed = ("X[i,j,q,r] = A[p,q,i] * B[r,j,p] | r,j,p,q,i ; Y[i,j,k,r] = X[i,j,q,r] * C[r,q,k] | r,j,q,k,i ; "
               "R[i,j,k] = Y[i,j,k,r] * D[r,j,k] | r,j,k,i")
    _, red = cst.schedule_check(printed, [("A", ("csf", (5, 6, 4))), ("B", ("csf", (8, 7, 5))),
                                          ("C", ("csf", (8, 6, 9))), ("D", ("csf", (8, 7, 9)))])
    assert red[:2] == [2, 2]
    # and with l bounded below what the fixed printed layouts allow, the search says so
    keep = [("A", ("csf", (5, 6, 4))), ("B", ("csf", (8, 7, 5))), ("C", ("csf", (8, 6, 9))), ("D", ("csf", (8, 7, 9)))]
    tree_printed = ("X[i,j,q,r] = A[p,q,i] * B[r,j,p] ; Y[i,j,k,r] = X[i,j,q,r] * C[r,q,k] ; "
                    "R[i,j,k] = Y[i,j,k,r] * D[r,j,k]")
    _, l_keep, _ = cst.schedule_search(tree_printed, keep, flags=cst.SEARCH_KEEP_LAYOUT)
    assert l_keep == 2
    with pytest.raises(cst.ConststnError):
        cst.schedule_search(tree_printed, keep, flags=cst.SEARCH_KEEP_LAYOUT, max_order=1)


def test_order5_chain_and_sparse_chain_trees():
    ops = [("X", ("csf", (3, 4, 5, 6, 7))), ("U4", (7, 2)), ("U3", (6, 2)), ("U2", (5, 2)), ("U1", (4, 2))]
    tree = ("T1[i,j,k,l,d] = X[i,j,k,l,m] * U4[m,d] ; T2[i,j,k,c,d] = T1[i,j,k,l,d] * U3[l,c] ; "
            "T3[i,j,b,c,d] = T2[i,j,k,c,d] * U2[k,b] ; Y[i,a,b,c,d] = T3[i,j,b,c,d] * U1[j,a]")
    text, l, _ = cst.schedule_search(tree, ops, flags=cst.SEARCH_KEEP_LAYOUT)
    _, red = cst.schedule_check(text, ops)
    assert max(red[:-1]) <= l <= 3                       # sharing only the sparse prefix would give 3; dense loops may lead too
    # the three-index transformation of Sec. 5.1, layouts free: order-1 workspace on (K,i)
    ops = [("I", ("csf", (9, 5, 5))), ("C", ("csf", (5, 3))), ("P", ("csf", (5, 4)))]
    text, l, modes = cst.schedule_search("T[K,i,v] = I[K,u,v] * C[u,i] ; E[K,i,m] = T[K,i,v] * P[v,m]", ops)
    assert l == 1


def test_what_the_search_refuses():
    X = ("X", ("csf", (5, 6, 7)))
    with pytest.raises(cst.ConststnError):               # loop orders already given
        cst.schedule_search(S.TTMC3, [X, ("U3", (7, 3)), ("U2", (6, 2))])
    with pytest.raises(cst.ConststnError):               # an operand used twice
        cst.schedule_search("T[i,j] = X[i,j,k] * v[k] ; z[i] = T[i,j] * v[j]", [X, ("v", (7,))])
    with pytest.raises(cst.ConststnError):               # two results: not a tree
        cst.schedule_search("T[i,j] = X[i,j,k] * v[k] ; S[i] = w[i] * u[i]", [X, ("v", (7,)), ("w", (5,)), ("u", (5,))])
