"""Comparison of a GPU speculative-decoding run with the oracle's run of the same inputs.

The two must agree token for token and decision for decision EXCEPT where the oracle flags the very
decision that differs: a draft token whose top-2 logit margin is below 2e-2, a halting decision whose
score lies within the stated distance of its threshold, or a target token (row of the verification
block) whose top-2 margin is below 2e-2.  Comparison stops at the first such position (what follows
depends on it); any other difference is an error.  No arithmetic of the method happens here."""
MARGIN = 2e-2


def first_difference(gi, oi):
    """Where two iteration records first differ: None, ("draft_token", j), ("halt", j) with j the 1-based draft
    step, or ("target_row", r)."""
    gb, ob = list(gi["block"]), list(oi["block"])
    assert gb[0] == ob[0], ("iterations start from different tokens", gb[0], ob[0])
    for j in range(1, min(len(gb), len(ob))):
        if gb[j] != ob[j]:
            return ("draft_token", j)
    if len(gb) != len(ob):
        return ("halt", min(len(gb), len(ob)) - 1 if min(len(gb), len(ob)) > 1 else 1)
    if gi["n"] != oi["n"] or list(gi["emit"]) != list(oi["emit"]):
        return ("target_row", min(gi["n"], oi["n"]))
    return None


def difference_is_flagged(diff, oi, halt_near=None):
    """halt_near(step_record) -> bool: the oracle's halting decision of that draft step lies within the stated
    distance of its threshold (None: the policy decides without floating point, so never)."""
    kind, idx = diff
    if kind == "draft_token":
        return oi["steps"][idx - 1]["margin"] < MARGIN
    if kind == "halt":
        # the shorter block stopped after step idx where the other went on: that step's decision differs; a
        # reference-lookahead block can also end one step earlier because the token of step idx + 1 differs
        steps = oi["steps"]
        cand = [s for s in (steps[idx - 1:idx + 1] if idx >= 1 else steps[:1])]
        return any((halt_near is not None and halt_near(s)) or s["margin"] < MARGIN for s in cand)
    if kind == "target_row":
        return oi["target_margins"][idx] < MARGIN
    raise ValueError(kind)


def compare_runs(gpu, orc, halt_near=None, on_equal=None):
    """Walks the iterations of both runs.  Returns the index of the iteration at which they diverged at a
    flagged decision (comparison stops there), or None if every iteration agrees.  An unflagged difference
    raises AssertionError.  on_equal(gi, oi) is called for every agreeing iteration."""
    for k, (gi, oi) in enumerate(zip(gpu["iterations"], orc["iterations"])):
        diff = first_difference(gi, oi)
        if diff is not None:
            assert difference_is_flagged(diff, oi, halt_near), (
                "iteration", k, diff, {x: gi[x] for x in ("sl", "n", "block", "emit")},
                {x: oi[x] for x in ("sl", "n", "block", "emit")})
            return k
        if on_equal is not None:
            on_equal(gi, oi)
    assert len(gpu["iterations"]) == len(orc["iterations"])
    return None
