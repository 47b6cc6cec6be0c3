"""Host-only tests of the C-ABI: exported symbols, layout planning, argument validation and the
state machine of a round (dry-run contexts make no GPU call, so these run without a GPU)."""
import ctypes as C
import os
import re

import pytest

import paper_1906_12043_amd as P
import synth_inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "cocod.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cocod_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"cocod_create", "cocod_local_steps", "cocod_average_begin", "cocod_average_end_apply",
            "cocod_destroy"} <= set(names)
    raw = C.CDLL(P.lib_path())
    for name in names:
        assert hasattr(raw, name), name
    assert P.lib().cocod_version() >= 1000


def test_config_struct_matches_header_size():
    # a wrong struct_size is refused, the right one gets past that check (and then fails on pointers)
    cfg = P.Config()
    cfg.struct_size = C.sizeof(P.Config) - 4
    out = C.c_void_p()
    assert P.lib().cocod_create(C.byref(cfg), C.byref(out)) == P.ERR_INVALID
    assert b"struct_size" in P.lib().cocod_last_error(None)
    cfg.struct_size = C.sizeof(P.Config)
    cfg.W, cfg.d, cfg.stride = 1, 4, 4
    assert P.lib().cocod_create(C.byref(cfg), C.byref(out)) == P.ERR_INVALID
    assert b"NULL" in P.lib().cocod_last_error(None)


# ---- layout --------------------------------------------------------------------------------

def expected_layout(sizes, bucket_bytes):
    """Tensors start on 1024-element (4 KiB) boundaries; the list's end is rounded up to 4 elements."""
    offsets, at = [], 0
    for n in sizes:
        at = (at + 1023) // 1024 * 1024
        offsets.append(at)
        at += n
    at = (at + 3) // 4 * 4
    cap = bucket_bytes // 4
    begins, start = [0], 0
    for t in range(1, len(sizes)):
        end = (offsets[t] + sizes[t] + 3) // 4 * 4
        if cap and end - start > cap:
            begins.append(offsets[t]); start = offsets[t]
    begins.append(at)
    return at, offsets, begins


def test_plan_layout_flat():
    assert P.plan_layout(65536) == (65536, [0], [0, 65536])
    assert P.plan_layout(10) == (12, [0], [0, 12])
    assert P.plan_layout(1) == (4, [0], [0, 4])


def test_plan_layout_bucketed_config():
    cfg = synth_inputs.CONFIGS["C5_bucketed"]
    sizes = synth_inputs.tensor_sizes(cfg["seed"], cfg["n_tensors"], cfg["d"], cfg["tensor_lo"], cfg["tensor_hi"])
    assert len(sizes) == 62 and sum(sizes) == cfg["d"]
    got = P.plan_layout(cfg["d"], sizes, cfg["bucket_bytes"])
    assert got == expected_layout(sizes, cfg["bucket_bytes"])
    padded, offsets, begins = got
    assert all(o % 1024 == 0 for o in offsets) and padded % 4 == 0 and padded - cfg["d"] <= 1023 * 61 + 3
    assert len(begins) - 1 >= 2                    # 44.8 MB of parameters in buckets of 25 MiB
    for a, b in zip(begins, begins[1:]):
        assert a in offsets and b > a


@pytest.mark.parametrize("sizes,bucket", [([5, 10, 3, 7], 48), ([1, 1, 1], 0), ([100, 1, 100], 16), ([4, 4, 4, 4], 32)])
def test_plan_layout_small_cases(sizes, bucket):
    assert P.plan_layout(sum(sizes), sizes, bucket) == expected_layout(sizes, bucket)


def test_plan_layout_errors():
    # the last two: d itself is in range, but the padded list (the second tensor starts on a 1024-element
    # boundary) passes 2^34 - 1024 elements = 2^24 - 1 chunks, the most one launch and 32-bit quad offsets take
    for d, sizes in [(0, None), (1 << 34, None), (10, [5, 4]), (10, [10, 0]), ((1 << 34) - 4, None),
                     ((1 << 34) - 1024, [1, (1 << 34) - 1025])]:
        with pytest.raises(P.CocodError) as e:
            P.plan_layout(d, sizes)
        assert e.value.status == P.ERR_INVALID


# ---- validation and state machine (dry run: pointers are never dereferenced) ----------------

def dry(**over):
    W, d = over.pop("W", 4), over.pop("d", 1000)
    stride = over.pop("stride", (d + 3) // 4 * 4)
    big = W * stride * 4
    base = 0x10000000
    kw = dict(W=W, d=d, stride=stride, lr=0.1, momentum=0.9, xA=base, xB=base + big, v=base + 2 * big,
              h=base + 3 * big, c=base + 4 * big, mean=base + 5 * big, flags=P.FLAG_DRY_RUN)
    kw.update(over)
    return P.Context(**kw)


@pytest.mark.parametrize("over,needle", [
    (dict(W=0), "W must"), (dict(W=70000), "W must"), (dict(d=0), "d must"),
    (dict(stride=996), "stride"), (dict(stride=1002), "stride"),
    (dict(xA=None), "NULL"), (dict(mean=None), "NULL"), (dict(v=None), "v must"), (dict(h=None), "h and c"),
    (dict(xA=0x10000004), "aligned"), (dict(xB=0x10000000), "overlap"),
    (dict(lr=float("nan")), "lr"), (dict(momentum=1.0), "momentum"), (dict(momentum=-0.1), "momentum"),
    (dict(weight_decay=-1.0), "weight_decay"), (dict(noise_sigma=-1.0), "noise_sigma"),
    (dict(weights=[0.5, 0.5, 0.5, 0.5]), "weights sum"), (dict(weights=[1.5, -0.5, 0, 0]), "weights["),
    (dict(noise_sigma_w=[0.1, -0.1, 0, 0]), "noise_sigma_w[1]"), (dict(noise_sigma_w=[0, 0, 0, float("inf")]), "noise_sigma_w[3]"),
    (dict(tensor_numel=[500, 400]), "sum to"), (dict(grad=7), "gradient kind"), (dict(flags=1 | 64), "flag"),
])
def test_create_rejects_bad_arguments(over, needle):
    with pytest.raises(P.CocodError) as e:
        dry(**over)
    assert e.value.status == P.ERR_INVALID and needle in str(e.value)


def test_momentum_zero_needs_no_v():
    with dry(momentum=0.0, v=None) as ctx:
        ctx.local_steps(2)


def test_round_state_machine_and_buffer_rotation():
    with dry() as ctx:
        a = ctx.live_model()
        assert not ctx.is_averaging() and ctx.get_step() == 0
        with pytest.raises(P.CocodError) as e:
            ctx.average_end_apply()
        assert e.value.status == P.ERR_STATE
        ctx.local_steps(3)                          # outside a round: in place
        assert ctx.live_model() == a and ctx.get_step() == 3
        ctx.average_begin()
        assert ctx.is_averaging()
        with pytest.raises(P.CocodError) as e:
            ctx.average_begin()
        assert e.value.status == P.ERR_STATE
        with pytest.raises(P.CocodError) as e:
            ctx.set_schedule(P.SCHED_SERIAL)
        assert e.value.status == P.ERR_STATE
        assert ctx.live_model() == a                # stored models are still the live ones
        ctx.local_steps(1)
        b = ctx.live_model()
        assert b != a                               # first step of the round went out of place
        ctx.local_steps(2)
        assert ctx.live_model() == b
        ctx.average_end_apply()
        assert not ctx.is_averaging() and ctx.live_model() == b and ctx.get_step() == 6
        ctx.round(2)
        assert ctx.live_model() == a and ctx.get_step() == 8
        ctx.average_begin(); ctx.average_end_apply()   # zero local steps: buffers do not rotate
        assert ctx.live_model() == a
        with pytest.raises(P.CocodError) as e:
            ctx.local_steps(-1)
        assert e.value.status == P.ERR_INVALID
        ctx.set_step(2**32 - 2)
        ctx.local_steps(1)
        with pytest.raises(P.CocodError):
            ctx.local_steps(1)
        with pytest.raises(P.CocodError):
            ctx.set_step(2**32)
        for s in (P.SCHED_OVERLAP, P.SCHED_SERIAL, P.SCHED_FUSED):
            ctx.set_schedule(s)
            ctx.set_step(0)
            ctx.round(1)
        with pytest.raises(P.CocodError):
            ctx.set_schedule(9)
        ctx.set_lr(0.01)
        with pytest.raises(P.CocodError):
            ctx.set_lr(float("inf"))


def test_plan_of_context():
    with dry(d=10000) as ctx:
        assert ctx.get_plan() == (10000, 10, 1)     # 9 x 1024 + 784
    sizes = [5000, 3, 4097]
    with dry(d=sum(sizes), tensor_numel=sizes, stride=10244, bucket_bytes=20480) as ctx:
        padded, chunks, buckets = ctx.get_plan()
        assert padded == 5120 + 1024 + 4100 and chunks == 5 + 1 + 5 and buckets == 3


def test_null_context_is_an_error_not_a_crash():
    L = P.lib()
    assert L.cocod_local_steps(None, 1) == P.ERR_INVALID
    assert L.cocod_average_begin(None) == P.ERR_INVALID
    assert L.cocod_average_end_apply(None) == P.ERR_INVALID
    assert L.cocod_sync(None) == P.ERR_INVALID
    assert L.cocod_destroy(None) == P.OK
    assert L.cocod_last_error(None) is not None


def test_local_steps_end_apply_state_machine():
    with dry() as ctx:
        with pytest.raises(P.CocodError) as e:
            ctx.local_steps_end_apply(2)
        assert e.value.status == P.ERR_STATE
        a = ctx.live_model()
        ctx.average_begin()
        ctx.local_steps_end_apply(3)
        assert not ctx.is_averaging() and ctx.get_step() == 3 and ctx.live_model() != a
        ctx.average_begin()
        ctx.local_steps_end_apply(0)
        assert not ctx.is_averaging() and ctx.get_step() == 3
        ctx.average_begin()
        with pytest.raises(P.CocodError) as e:
            ctx.local_steps_end_apply(-1)
        assert e.value.status == P.ERR_INVALID and ctx.is_averaging()
        ctx.local_steps_end_apply(1)
        assert not ctx.is_averaging() and ctx.get_step() == 4


def test_external_step_state_machine():
    g = 0x70000000
    with dry(grad=P.GRAD_EXTERNAL, h=None, c=None) as ctx:
        for call in (lambda: ctx.local_steps(1), lambda: ctx.local_steps_end_apply(1)):
            ctx.average_begin() if not ctx.is_averaging() else None
            with pytest.raises(P.CocodError) as e:
                call()
            assert e.value.status == P.ERR_INVALID and "external" in str(e.value)
        ctx.local_steps(0)                               # zero steps need no gradient
        a = ctx.live_model()
        ctx.external_step(g)
        assert ctx.live_model() != a and ctx.get_step() == 1 and ctx.is_averaging()
        ctx.external_step(g, close_round=True)
        assert not ctx.is_averaging() and ctx.get_step() == 2
        with pytest.raises(P.CocodError) as e:
            ctx.external_step(g, close_round=True)
        assert e.value.status == P.ERR_STATE
        for bad in (None, g + 4):
            with pytest.raises(P.CocodError) as e:
                ctx.external_step(bad)
            assert e.value.status == P.ERR_INVALID
        ctx.external_step(g)                             # outside a round: plain SGD step
        assert ctx.get_step() == 3
        ctx.external_step_bf16(g + 8)                    # 16-bit gradients need 8-byte alignment only
        assert ctx.get_step() == 4
        for bad in (None, g + 4):
            with pytest.raises(P.CocodError) as e:
                ctx.external_step_bf16(bad)
            assert e.value.status == P.ERR_INVALID
        ctx.average_begin()
        ctx.external_step_bf16(g, close_round=True)
        assert not ctx.is_averaging() and ctx.get_step() == 5
    with dry() as ctx:                                  # also legal on a context with a built-in gradient
        ctx.external_step(g)
        assert ctx.get_step() == 1


FAKE_STREAM = 0x40                 # dry-run contexts never touch their streams


def test_graph_round_needs_a_capturable_stream():
    for stream in (None, 1):                              # the null stream and the legacy default-stream handle
        with dry(compute_stream=stream) as ctx:
            with pytest.raises(P.CocodError) as e:
                ctx.graph_round(1)
            assert e.value.status == P.ERR_INVALID and "null stream" in str(e.value)
            assert ctx.get_step() == 0 and not ctx.is_averaging()


def test_average_apply_fused_state_machine():
    with dry() as ctx:
        a = ctx.live_model()
        ctx.average_apply_fused()                         # idle: blocking average, nothing rotates
        assert not ctx.is_averaging() and ctx.live_model() == a and ctx.get_step() == 0
        for sched in (P.SCHED_OVERLAP, P.SCHED_SERIAL, P.SCHED_FUSED, P.SCHED_HEAD):
            ctx.set_schedule(sched)
            ctx.average_begin()
            ctx.local_steps(2)
            ctx.average_apply_fused()                     # closes the open round under every schedule
            assert not ctx.is_averaging()
            with pytest.raises(P.CocodError) as e:
                ctx.average_end_apply()
            assert e.value.status == P.ERR_STATE
        assert ctx.get_step() == 8
    assert P.lib().cocod_average_apply_fused(None) == P.ERR_INVALID      # NULL context: an error, not a crash


def test_graph_round_state_machine():
    with dry(compute_stream=FAKE_STREAM, avg_stream=FAKE_STREAM) as ctx:
        a = ctx.live_model()
        ctx.graph_round(3, fused_tail=True)
        assert ctx.get_step() == 3 and not ctx.is_averaging() and ctx.live_model() != a
        ctx.graph_round(2, fused_tail=False)
        assert ctx.get_step() == 5 and ctx.live_model() == a
        ctx.graph_round(0)                                   # pure averaging: no buffer swap, no step
        assert ctx.get_step() == 5 and ctx.live_model() == a
        ctx.average_begin()
        with pytest.raises(P.CocodError) as e:
            ctx.graph_round(1)
        assert e.value.status == P.ERR_STATE
        ctx.average_end_apply()
        with pytest.raises(P.CocodError) as e:
            ctx.graph_round(-1)
        assert e.value.status == P.ERR_INVALID
    with dry(grad=P.GRAD_EXTERNAL, h=None, c=None, compute_stream=FAKE_STREAM) as ctx:
        with pytest.raises(P.CocodError) as e:
            ctx.graph_round(1)
        assert e.value.status == P.ERR_INVALID
        ctx.graph_round(0)


def test_diagnostics_on_dry_contexts():
    with dry() as ctx:
        assert ctx.consensus_distance() == 0.0 and ctx.quadratic_objective() == (0.0, 0.0)
    with dry(grad=P.GRAD_EXTERNAL, h=None, c=None) as ctx:
        with pytest.raises(P.CocodError) as e:
            ctx.quadratic_objective()
        assert e.value.status == P.ERR_INVALID


def test_launch_size_limits():
    """One block per (chunk of 1024 elements, worker): the product must fit a launch."""
    with pytest.raises(P.CocodError) as e:
        dry(W=65535, d=2**34 - 1024)
    assert e.value.status == P.ERR_INVALID and "too large" in str(e.value)
    with pytest.raises(P.CocodError) as e:
        dry(W=2048, d=2**30 + 1024)                       # 2^20 + 1 chunks x 2^11 workers > 2^31 - 1
    assert e.value.status == P.ERR_INVALID
    with dry(W=2047, d=2**30) as ctx:                      # 2^20 chunks x 2047 workers: fits
        assert ctx.get_plan() == (2**30, 2**20, 1)
        ctx.round(2)
        ctx.round_fused_tail(1)


def test_plain_c_client_of_the_abi(tmp_path):
    """The header is C (compiled -std=c99 -pedantic, warnings are errors) and the library is usable from a
    C program with no Python in between: tests/c_abi_client.c walks a dry-run context."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    exe = str(tmp_path / "c_abi_client")
    libdir = os.path.dirname(P.lib_path())
    build = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                            os.path.join(ROOT, "tests", "c_abi_client.c"), "-o", exe, "-L", libdir, "-lcocod",
                            "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert run.returncode == 0 and "c abi client: ok" in run.stdout, run.stderr


def test_no_alloc_consensus_distance_limits_on_the_host():
    """The static scratch holds 2^18 block partials: a larger model is refused with a clear error (dry-run
    contexts: no GPU call), a model at the limit is accepted."""
    with dry(W=2, d=2**28) as ctx:                        # exactly 2^18 chunks
        ctx.consensus_distance_noalloc(0x1000)
    with dry(W=2, d=2**28 + 1) as ctx:
        with pytest.raises(P.CocodError) as e:
            ctx.consensus_distance_noalloc(0x1000)
        assert e.value.status == P.ERR_UNSUPPORTED and "exceed the static scratch" in str(e.value)
    with dry() as ctx:
        with pytest.raises(P.CocodError) as e:
            ctx.consensus_distance_noalloc(None)
        assert e.value.status == P.ERR_INVALID
