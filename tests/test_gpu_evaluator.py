"""The evaluator has no ground truth in the paper; it is judged by how well its ranking of the
enumerated candidates agrees with measured times: AUTO's pick must be close to the measured best."""
import pytest

from tests.gpu_util import note
from workloads import FULL_CONFIGS, GENERIC_CONFIGS, NEXT_CONFIGS

pytestmark = pytest.mark.gpu


def _time_candidates(cfg, steps, only_generated=False):
    import torch
    from bench import Runner
    from paper_2009_10924_amd import binding as B
    spec = dict(FULL_CONFIGS, **GENERIC_CONFIGS, **NEXT_CONFIGS)[cfg]()
    plan = B.Plan(B.Graph.from_spec(spec), "auto")
    cands = plan.candidates()
    host, rows = None, []
    for i, ci in enumerate(cands):
        if only_generated and ci["pattern"] != "row_generated":
            continue                                    # the interpreted forms are fallbacks, not rivals
        try:
            r = Runner(spec, "auto", host_inputs=host, candidate=i)
        except B.FsError as e:
            assert "scratch memory" in e.text           # a shape the compiled kernel cannot hold in registers
            continue
        if only_generated and i == plan.info["candidate"]:
            ci = dict(ci, predicted_us=-1.0)            # marks AUTO's own pick (made after compiling, with real registers)
        host = r.host_inputs
        _, ev = r.time_region(steps, 20)
        rows.append((ev / steps * 1e6, ci["predicted_us"], ci["kernel"]))
        del r
        torch.cuda.empty_cache()
    return rows


@pytest.mark.parametrize("cfg,steps", [("C2", 600), ("C3", 600), ("C4", 100), ("C5", 150), ("N2", 300)])
def test_auto_pick_is_near_the_measured_best(cfg, steps):
    rows = _time_candidates(cfg, steps)
    best = min(r[0] for r in rows)
    pick = min(rows, key=lambda r: r[1])
    for us, pred, name in rows:
        note(f"    {cfg} {name:44s} measured {us:8.2f} us predicted {pred:8.2f} us")
    note(f"  {cfg}: picked {pick[2]} at {pick[0]:.2f} us, best {best:.2f} us")
    assert pick[0] <= 1.10 * best, f"{cfg}: evaluator's choice is {pick[0] / best - 1:.1%} slower than the best candidate"
    # the worst candidate must not be predicted best-or-near-best: ranking carries information
    worst = max(rows, key=lambda r: r[0])
    assert worst[1] > min(r[1] for r in rows)
    if cfg == "C2":
        # the choice between warp composition and block composition (reduced values through LDS) is part of what is
        # judged: both kinds are among the timed candidates
        assert any("layernorm_block" in r[2] for r in rows) and any("layernorm_wave" in r[2] for r in rows)


@pytest.mark.parametrize("cfg,steps", [("G1", 300), ("G4", 300), ("G6", 150), ("G9", 100), ("G10", 100), ("G11", 20), ("G12", 20)])
def test_auto_pick_among_generated_shapes_is_near_the_measured_best(cfg, steps):
    """The same judgement for the shapes of a generated kernel (lanes per row, steps per lane, step width, rows per
    lane group, column tiles): what AUTO compiles and runs is within 10 % of the fastest shape."""
    from paper_2009_10924_amd import binding as B
    if not B.codegen_available():
        pytest.skip("needs the run-time compiler")
    rows = _time_candidates(cfg, steps, only_generated=True)
    best = min(r[0] for r in rows)
    pick = [r for r in rows if r[1] < 0][0]
    for us, pred, name in rows:
        note(f"    {cfg} {name:56s} measured {us:8.2f} us {'<- AUTO' if pred < 0 else f'predicted {pred:8.2f} us'}")
    assert pick[0] <= 1.10 * best, f"{cfg}: AUTO's shape is {pick[0] / best - 1:.1%} slower than the best one"
