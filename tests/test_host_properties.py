"""Property tests of the host logic (no GPU): the layout planner against an independent restatement,
and random walks over the round's state machine (dry-run contexts) against a small Python model."""
import random

import pytest
from hypothesis import given, settings, strategies as st

import paper_1906_12043_amd as P


def model_layout(sizes, bucket_bytes):
    """Restated from the layout rules: tensors in order, each start on a multiple of 1024 elements, end of
    the list rounded up to 4; a bucket is a maximal run of tensors whose extent (first start to the end of
    the last, rounded up to 4) fits bucket_bytes."""
    offsets, at = [], 0
    for n in sizes:
        at = -(-at // 1024) * 1024
        offsets.append(at)
        at += n
    padded = -(-at // 4) * 4
    begins = [0]
    if bucket_bytes:
        start = 0
        for t in range(1, len(sizes)):
            end = -(-(offsets[t] + sizes[t]) // 4) * 4
            if (end - start) * 4 > bucket_bytes:
                begins.append(offsets[t])
                start = offsets[t]
    begins.append(padded)
    return padded, offsets, begins


@settings(max_examples=200, deadline=None)
@given(st.lists(st.integers(1, 5000), min_size=2, max_size=12), st.sampled_from([0, 16, 4096, 10000, 40000, 1 << 20]))
def test_layout_planner_matches_the_restated_rules(sizes, bucket_bytes):
    got = P.plan_layout(sum(sizes), sizes, bucket_bytes)
    assert got == model_layout(sizes, bucket_bytes)
    padded, offsets, begins = got
    # tensors do not overlap, buckets partition [0, padded) at tensor starts
    for a, n, b in zip(offsets, sizes, offsets[1:] + [padded]):
        assert a % 1024 == 0 and a + n <= b
    assert begins[0] == 0 and begins[-1] == padded and begins == sorted(set(begins))
    assert all(b in offsets for b in begins[:-1])


class RoundModel:
    """What the calls do to the observable state: step counter, which buffer is live, whether a round is open."""

    def __init__(self):
        self.step, self.live_is_a, self.open, self.first = 0, True, False, False

    def steps(self, k):
        if k > 0 and self.first:
            self.live_is_a = not self.live_is_a
            self.first = False
        self.step += k

    def begin(self):
        self.open, self.first = True, True

    def end(self):
        self.open, self.first = False, False


@pytest.mark.parametrize("seed", range(8))
def test_random_walk_over_the_state_machine(seed):
    rng = random.Random(seed)
    base = 0x10000000
    W, d = 3, 2000
    big = W * d * 4
    ctx = P.Context(W=W, d=d, stride=d, lr=0.1, momentum=0.9, xA=base, xB=base + big, v=base + 2 * big, h=base + 3 * big,
                    c=base + 4 * big, mean=base + 5 * big, flags=P.FLAG_DRY_RUN,
                    compute_stream=0x40, avg_stream=0x40)          # never touched by a dry-run context; graph rounds refuse the null stream
    m = RoundModel()
    g = base + 6 * big
    for _ in range(400):
        op = rng.choice(["steps", "begin", "end", "tail", "ext", "ext_close", "graph", "sched", "lr", "fused"])
        k = rng.choice([0, 0, 1, 1, 2, 3])
        try:
            if op == "steps":
                ctx.local_steps(k); m.steps(k)
            elif op == "begin":
                ctx.average_begin(); assert not m.open; m.begin()
            elif op == "end":
                ctx.average_end_apply(); assert m.open; m.end()
            elif op == "tail":
                ctx.local_steps_end_apply(k); assert m.open; m.steps(k); m.end()
            elif op == "ext":
                ctx.external_step(g); m.steps(1)
            elif op == "ext_close":
                ctx.external_step_bf16(g, close_round=True); assert m.open; m.steps(1); m.end()
            elif op == "graph":
                fused = rng.random() < 0.5
                ctx.graph_round(k, fused); assert not m.open; m.begin(); m.steps(k); m.end()
            elif op == "fused":                               # closes an open round, or is a blocking average while idle
                ctx.average_apply_fused()
                if m.open:
                    m.end()
            elif op == "sched":
                ctx.set_schedule(rng.choice([P.SCHED_OVERLAP, P.SCHED_SERIAL, P.SCHED_FUSED, P.SCHED_HEAD])); assert not m.open
            else:
                ctx.set_lr(rng.choice([0.1, 0.05]))
        except P.CocodError as e:
            # the only legal refusals in this walk are state errors, and only where the model agrees
            assert e.status == P.ERR_STATE, (op, str(e))
            assert (op in ("begin", "graph", "sched")) == m.open and (op in ("end", "tail", "ext_close")) == (not m.open), (op, m.open)
        assert ctx.get_step() == m.step
        assert ctx.is_averaging() == m.open
        assert (ctx.live_model() == base) == m.live_is_a
    ctx.close()
