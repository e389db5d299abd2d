"""Pins for the oracle's draft verification and the expected-speed-up formula (arXiv 2503.13565,
sections 3.1 to 3.3, Eq. 1).  The accept rule is checked against a brute-force statement of
"drop everything after the first mismatch" on every small case; the formula against the numbers
and ranges the paper gives in its text.
"""
import itertools

import numpy as np
import pytest

import oracle


def test_accept_matches_brute_force_on_every_small_case():
    vocab = (3, 5, 7)
    for n in range(0, 5):
        for target in itertools.product(vocab, repeat=n + 1):
            for draft in itertools.product(vocab, repeat=n):
                emitted = []                                  # tokens this round puts out, by the text
                for m in range(n):
                    if draft[m] != target[m]:
                        break
                    emitted.append(draft[m])
                emitted.append(target[len(emitted)])
                g, nxt = oracle.greedy_accept(target, draft)
                assert g == len(emitted) - 1 and nxt == emitted[-1], (target, draft)
                assert 0 <= g <= n


def test_accept_special_cases():
    assert oracle.greedy_accept([9], []) == (0, 9)                       # no drafts: plain greedy step
    assert oracle.greedy_accept([1, 2, 3, 4], [1, 2, 3]) == (3, 4)       # all accepted + the extra token
    assert oracle.greedy_accept([1, 2, 3, 4], [8, 2, 3]) == (0, 1)       # later matches do not count
    assert oracle.greedy_accept([1, 2, 3, 4], [1, 8, 3]) == (1, 2)


def test_eq1_both_forms_agree_and_match_the_text():
    for n in (1, 2, 4, 8):
        for g in range(n + 1):
            for s in (1.5, 4.0, 20.0, 100.0):
                a = oracle.sd_speedup(g, n, s)
                b = oracle.sd_speedup_alpha(g / n, n, s)
                assert a == pytest.approx(b, rel=1e-14)
    # the text's instance of Eq. 1 for N = 4: (alpha + 0.25) / (1 / S + 0.25)
    for alpha in (0.0, 0.417, 0.712, 0.9, 1.0):
        for s in (4.0, 20.0, 100.0):
            assert oracle.sd_speedup_alpha(alpha, 4, s) == pytest.approx((alpha + 0.25) / (1 / s + 0.25), rel=1e-14)
    # limits: nothing accepted with a free draft gives 1 token per target run; a draft as slow as
    # the target with everything accepted gives (N + 1) / (N + 1)
    assert oracle.sd_speedup(0, 4, 1e300) == pytest.approx(1.0)
    assert oracle.sd_speedup(4, 4, 1.0) == pytest.approx(1.0)
    assert oracle.sd_speedup(4, 4, 1e300) == pytest.approx(5.0)


def test_paper_ranges_section_3_2_and_3_3():
    # section 3.2: a 4x faster draft at 80-90 % acceptance is on a par with 20x / 100x faster
    # drafts at about half that acceptance
    q = [oracle.sd_speedup_alpha(a, 4, 4.0) for a in (0.8, 0.9)]
    tiny = [oracle.sd_speedup_alpha(a, 4, s) for a in (0.4, 0.45) for s in (20.0, 100.0)]
    assert 2.0 <= min(q) and max(q) <= 2.5
    assert 2.0 <= min(tiny) and max(tiny) <= 2.75
    # section 3.3: 80-85 % for the 4-bit draft and 40-45 % for the tiny (100x) draft give about
    # 3-3.5x in two levels, against 2-2.5x for either draft alone
    two = [oracle.sd_speedup_two_level(am, 4, 4.0, al, 4, 100.0) for am in (0.8, 0.85) for al in (0.4, 0.45)]
    assert 2.85 <= min(two) and max(two) <= 3.5
    for am in (0.8, 0.85):
        for al in (0.4, 0.45):
            t = oracle.sd_speedup_two_level(am, 4, 4.0, al, 4, 100.0)
            assert t > oracle.sd_speedup_alpha(am, 4, 4.0) and t > oracle.sd_speedup_alpha(al, 4, 100.0)
    # the composition by hand for one point
    s_prime = 4.0 * (0.45 + 0.25) / (0.25 + 1 / 25.0)
    assert oracle.sd_speedup_two_level(0.85, 4, 4.0, 0.45, 4, 100.0) == pytest.approx((0.85 + 0.25) / (0.25 + 1 / s_prime))
