"""The planner's choices against the clock: every candidate of every stage that leaves a choice (first product: kernel
and ranges of d; down projection: ffn ranges; last product: tile size) is forced in turn through svdmlp_force_plan and
timed with the library's per-kernel events; the candidate the cost model picks must be within a few percent of the
fastest one (the counterpart of the block-size sweep of the paper's Sec. 5.3, Table 3, where the model of Eq. 10 - 11
picks the block)."""
import re
import statistics

import pytest
import torch

from paper_2510_25977_amd import binding as B
from paper_2510_25977_amd import synth

pytestmark = pytest.mark.gpu

STEPS = 30


def kernel_times_us(mlp, X, Y):
    for _ in range(6):
        mlp(X, Y)
    torch.cuda.synchronize()
    runs = []
    for _ in range(3):
        B.svdmlp_profile_begin(mlp.ctx, STEPS)
        for _ in range(STEPS):
            mlp(X, Y)
        k, _ = B.svdmlp_profile_end(mlp.ctx)
        runs.append(k)
    return {n: statistics.median(r[n] for r in runs) * 1e3 for n in runs[0]}


def time_every_candidate(mlp, X, Y, text):
    """Per stage: the time of the candidate the planner chose and of every other candidate, all forced through
    svdmlp_force_plan and timed under the same conditions."""
    for _ in range(60):                       # let the clocks settle before anything is compared
        mlp(X, Y)
    auto = kernel_times_us(mlp, X, Y)
    first_name = "k_in" if "k_in" in auto else "k_s1"
    last_name = "k_out" if "k_out" in auto else "k_s5"
    # what the planner chose, from its own description
    m = re.search(r"k_(s1|in)\[tile=\S+ tiles=\d+ ranges=(\d+)", text)
    chosen_first = (B.FIRST_IN if m.group(1) == "in" else B.FIRST_S1, int(m.group(2)))
    chosen_down = int(re.search(r"k_down1\[tile=\S+ tiles=\d+ ranges=(\d+)", text).group(1))
    chosen_out = B.OUT_256 if re.search(r" k_out\[", text) else B.OUT_128
    assert first_name == ("k_in" if chosen_first[0] == B.FIRST_IN else "k_s1")
    assert last_name == ("k_out" if chosen_out == B.OUT_256 else "k_s5")
    first, down, out = {}, {}, {}
    for kern in (B.FIRST_S1, B.FIRST_IN):
        for S in sorted({1, 2, 3, 4, 6, 8, chosen_first[1]}):
            B.svdmlp_force_plan(mlp.ctx, kern, S, 0, 0)
            k = kernel_times_us(mlp, X, Y)
            ran = "k_in" if "k_in" in k else "k_s1"
            if (ran == "k_in") != (kern == B.FIRST_IN):
                continue          # not a valid candidate at these extents: the planner's own choice ran
            first[(kern, S)] = k[ran]
    for s_ in sorted({1, 2, 4, 6, 8, 12, 16, 24, 32, chosen_down}):
        B.svdmlp_force_plan(mlp.ctx, 0, 0, s_, 0)
        k = kernel_times_us(mlp, X, Y)
        down[s_] = k["k_down1"] + k.get("k_reduce", 0.0)
    for o in (B.OUT_256, B.OUT_128):
        B.svdmlp_force_plan(mlp.ctx, 0, 0, 0, o)
        k = kernel_times_us(mlp, X, Y)
        ran = "k_out" if "k_out" in k else "k_s5"
        if (ran == "k_out") != (o == B.OUT_256):
            continue
        out[o] = k[ran]
    B.svdmlp_force_plan(mlp.ctx, 0, 0, 0, 0)
    again = kernel_times_us(mlp, X, Y)
    assert set(again) == set(auto)                      # the override is gone
    chosen = {"first": first[chosen_first], "down": down[chosen_down], "out": out[chosen_out]}
    best = {"first": min(first.values()), "down": min(down.values()), "out": min(out.values())}
    tried = {"first": len(first), "down": len(down), "out": len(out)}
    return chosen, best, tried


def plan_is_good(chosen, best):
    """Per stage within 10 % (+ 0.5 us of timer noise) of the fastest candidate; the three stages together within 5 %."""
    return (all(chosen[s] <= 1.10 * best[s] + 0.5 for s in chosen)
            and sum(chosen.values()) <= 1.05 * sum(best.values()) + 0.5)


@pytest.mark.parametrize("name,kw", [("prefill", dict(r=256)), ("prefill", dict(r=512)), ("prefill", dict(r=1024)),
                                     ("wide", {}), ("mlp_small", {})])
def test_chosen_plan_is_within_five_percent_of_the_best_candidate(name, kw):
    gi = synth.make_workload(name, **kw)
    dm = gi.dims
    dev = torch.device("cuda:0")
    f = {k: v.to(dev) for k, v in gi.factors().items()}
    mlp = B.SvdMlp(max_M=dm["M"], flags=B.FLAG_PLAN_ROOM | B.FLAG_FORCE_TILED, keep_factors=False, **f)
    X = gi.X.to(dev)
    Y = torch.empty_like(X)
    text = B.svdmlp_describe(mlp.desc, dm["M"])
    # kernel times on a shared machine jitter by a few percent from one minute to the next: a sweep that misses the
    # bar is repeated (up to three in all) and the last one decides
    for attempt in range(3):
        chosen, best, tried = time_every_candidate(mlp, X, Y, text)
        if plan_is_good(chosen, best):
            break
    mlp.close()
    assert tried["first"] >= 4 and tried["down"] >= 6 and tried["out"] >= 1, tried
    assert plan_is_good(chosen, best), (chosen, best, text)
    # the model's estimate of what it chose is in the right place (it ranks candidates; it is not a simulator)
    est = [float(x) for x in re.findall(r"est_us=([0-9.]+)", text)]
    assert len(est) == 3
    for e, stage in zip(est, ("first", "down", "out")):
        assert 0.5 * chosen[stage] <= e <= 1.6 * chosen[stage], (stage, e, chosen)


def test_forced_candidates_compute_the_same_result():
    """Whatever candidate runs, the forward is the same function: outputs of forced plans against the automatic one
    (different contraction cuts add in a different order, so equal up to fp32 summation order, then bf16 rounding)."""
    gi = synth.make_gated(700, 1024, 4096, 256, 512, stream=83)
    dev = torch.device("cuda:0")
    f = {k: v.to(dev) for k, v in gi.factors().items()}
    mlp = B.SvdMlp(max_M=700, flags=B.FLAG_PLAN_ROOM | B.FLAG_FORCE_TILED, **f)
    X = gi.X.to(dev)
    ref = mlp(X).float()
    scale = float(ref.abs().max())
    for plan in ((B.FIRST_S1, 1, 1, B.OUT_128), (B.FIRST_S1, 2, 3, B.OUT_256), (B.FIRST_IN, 1, 7, 0), (B.FIRST_IN, 2, 32, B.OUT_256),
                 (0, 0, 16, B.OUT_128)):
        B.svdmlp_force_plan(mlp.ctx, *plan)
        Y = mlp(X).float()
        torch.cuda.synchronize()
        assert float((Y - ref).abs().max()) <= 1e-2 * scale, plan
    # without SVDMLP_FLAG_PLAN_ROOM a forced candidate either fits the partial-sum buffer the planner's own choices
    # need (then it runs and gives the same result) or the forward refuses it loudly; never a silent overrun
    tight = B.SvdMlp(max_M=700, flags=B.FLAG_FORCE_TILED, **f)
    B.svdmlp_force_plan(tight.ctx, 0, 0, 32, 0)
    try:
        Y = tight(X).float()
        torch.cuda.synchronize()
        assert float((Y - ref).abs().max()) <= 1e-2 * scale
    except B.SvdMlpError as e:
        assert e.status == B.SVDMLP_HIP_ERROR
    B.svdmlp_force_plan(tight.ctx, 0, 0, 0, 0)
    Y = tight(X).float()
    torch.cuda.synchronize()
    assert torch.equal(Y, ref)
    tight.close()
    mlp.close()
