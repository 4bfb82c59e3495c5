"""The format planner of the layer stack is pure host logic (a dynamic program over measured times): checked here on
hand-made timing tables against exhaustive enumeration and against cases whose answer is obvious."""
import itertools

import pytest

from paper_1611_06945_amd.stack import NCHW, NHWC, plan_formats

INF = float("inf")


def brute_force(conv_t, fused_t, glue_t, x_cvt):
    """Every assignment of (format, output layout, fused) per layer, costed directly."""
    n = len(conv_t)
    options = []
    for i in range(n):
        o = [(fmt, olay, False, t) for (fmt, olay), t in conv_t[i].items()]
        o += [(fmt, olay, True, t) for (fmt, olay), t in fused_t[i].items()]
        options.append(o)
    best = (INF, None)
    for pick in itertools.product(*options):
        total = x_cvt if pick[0][0] == NHWC else 0.0
        ok = True
        for i, (fmt, olay, fz, t) in enumerate(pick):
            want = pick[i + 1][0] if i + 1 < n else NCHW   # what the next layer reads; the stack hands on planar tensors
            total += t
            if fz:
                ok = ok and olay == want
            else:
                total += glue_t[i][(olay, want)]
        if ok and total < best[0]:
            best = (total, pick)
    return best


def tables(n, pooled, seed):
    import random

    rnd = random.Random(seed)
    conv_t, fused_t, glue_t = [], [], []
    for i in range(n):
        c = {(NCHW, NCHW): rnd.uniform(5, 30)}
        if rnd.random() < 0.8:
            c[(NHWC, NHWC)] = rnd.uniform(3, 30)
            c[(NHWC, NCHW)] = rnd.uniform(3, 30)
        if rnd.random() < 0.4:
            c[(NCHW, NHWC)] = rnd.uniform(5, 30)
        f = {}
        if i in pooled and rnd.random() < 0.7:
            for key in list(c):
                if rnd.random() < 0.6:
                    f[key] = c[key] + rnd.uniform(-2, 6)
        if i in pooled:
            g = {(a, b): rnd.uniform(2, 6) for a in (NCHW, NHWC) for b in (NCHW, NHWC)}
        else:
            g = {(a, b): (0.0 if a == b else rnd.uniform(2, 8)) for a in (NCHW, NHWC) for b in (NCHW, NHWC)}
        conv_t.append(c)
        fused_t.append(f)
        glue_t.append(g)
    return conv_t, fused_t, glue_t


@pytest.mark.parametrize("seed", range(40))
def test_plan_is_the_cheapest_assignment(seed):
    n = 2 + seed % 4
    conv_t, fused_t, glue_t = tables(n, pooled={0, 1, n - 1} if seed % 2 else {1}, seed=seed)
    x_cvt = INF if seed % 5 == 0 else 3.0 + seed % 3
    chosen, olays, fused, total = plan_formats(conv_t, fused_t, glue_t, x_cvt)
    want_total, pick = brute_force(conv_t, fused_t, glue_t, x_cvt)
    assert total == pytest.approx(want_total)
    # the returned assignment really costs what the planner says
    cost = x_cvt if chosen[0] == NHWC else 0.0
    for i in range(n):
        nxt = chosen[i + 1] if i + 1 < n else NCHW
        if fused[i]:
            assert olays[i] == nxt and (chosen[i], olays[i]) in fused_t[i]
            cost += fused_t[i][(chosen[i], olays[i])]
        else:
            cost += conv_t[i][(chosen[i], olays[i])] + glue_t[i][(olays[i], nxt)]
    assert cost == pytest.approx(total)


def test_everything_planar_when_nothing_else_exists():
    conv_t = [{(NCHW, NCHW): 10.0}, {(NCHW, NCHW): 20.0}]
    glue_t = [{(a, b): (0.0 if a == b else 5.0) for a in (NCHW, NHWC) for b in (NCHW, NHWC)}] * 2
    assert plan_formats(conv_t, [{}, {}], glue_t, INF) == ([NCHW, NCHW], [NCHW, NCHW], [False, False], 30.0)


def test_a_fused_pool_wins_only_when_it_is_cheaper_than_convolution_plus_pool():
    glue = {(a, b): 4.0 for a in (NCHW, NHWC) for b in (NCHW, NHWC)}       # a pool behind layer 0
    last = {(a, b): (0.0 if a == b else 3.0) for a in (NCHW, NHWC) for b in (NCHW, NHWC)}
    conv_t = [{(NCHW, NCHW): 13.0}, {(NHWC, NCHW): 9.0, (NCHW, NCHW): 15.0}]
    cheap = plan_formats(conv_t, [{(NCHW, NHWC): 12.5}, {}], [glue, last], INF)
    assert cheap == ([NCHW, NHWC], [NHWC, NCHW], [True, False], 21.5)
    dear = plan_formats(conv_t, [{(NCHW, NHWC): 18.0}, {}], [glue, last], INF)
    assert dear == ([NCHW, NHWC], [NCHW, NCHW], [False, False], 26.0)   # 13 + pool 4 (converting) + 9


def test_the_last_layer_hands_on_planar_tensors():
    glue = {(a, b): (0.0 if a == b else 2.0) for a in (NCHW, NHWC) for b in (NCHW, NHWC)}
    chosen, olays, fused, total = plan_formats([{(NHWC, NHWC): 5.0, (NCHW, NCHW): 9.0}], [{}], [glue], 1.0)
    assert (chosen, olays, fused, total) == ([NHWC], [NHWC], [False], 8.0)   # 1 (input) + 5 + 2 (back to planar)


def test_an_impossible_chain_is_reported():
    with pytest.raises(ValueError):
        plan_formats([{}], [{}], [{}], INF)
