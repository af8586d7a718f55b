"""Host-only checks of the C ABI: the library loads, exports every declared symbol, plans
networks and rejects bad arguments before touching a device.  No GPU needed."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2102_13243_amd import binding as B
from workloads import nets

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "s4tf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(s4tf_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_symbols()
    assert "s4tf_train_step" in names and "s4tf_conv2d_vjp" in names and len(names) >= 20
    for n in names:
        assert hasattr(L, n), n


def test_binding_has_the_same_names():
    for n in declared_symbols():
        if n in ("s4tf_last_error", "s4tf_profile_class_name"):
            continue
        assert hasattr(B, n), n


@pytest.mark.parametrize("name,expect", [("tiny", 634), ("lenet5", 61706), ("resnet56", 855770),
                                         ("resnet50", 25557032), ("mobilenetv2", 3504872)])
def test_net_planning_matches_parameter_counts(name, expect):
    net = nets.CONFIGS[name]()
    desc, keep = B.make_net_desc(net)
    off, size = B.s4tf_net_param_layout(desc)
    assert sum(size) == expect
    count = B.s4tf_net_param_count(desc)
    assert count >= expect and count % 8 == 0
    # tensors do not overlap, start at multiples of 8 elements, and are in op order
    spans = sorted((o, s) for o, s in zip(off, size) if s)
    for (o1, s1), (o2, _) in zip(spans, spans[1:]):
        assert o1 % 8 == 0 and o1 + s1 <= o2
    assert B.s4tf_train_step_workspace_bytes(desc) > 0


def test_lenet_plan_follows_paper_shapes():
    # fc1 has inputSize 400 in the paper's LeNet figure: the planner must derive 16*5*5
    net = nets.lenet5()
    desc, keep = B.make_net_desc(net)
    _, size = B.s4tf_net_param_layout(desc)
    assert size[2 * 5] == 400 * 120 and size[2 * 5 + 1] == 120
    assert size[0] == 5 * 5 * 1 * 6 and size[2 * 2] == 5 * 5 * 6 * 16


def test_bad_arguments_are_rejected_on_the_host():
    L = B.lib()
    d = B.ConvDesc(1, 8, 8, 4, 4, 3, 3, 1, 1, 1, B.S4TF_F32, 0, 0)
    assert L.s4tf_conv2d_fwd(ctypes.byref(d), None, None, None, None, None, 0, None) == -1
    assert "NULL" in B.last_error()
    assert L.s4tf_conv2d_fwd(ctypes.byref(d), 8, 16, None, 16, None, 0, None) == -7      # misaligned x
    bad = B.ConvDesc(1, 8, 8, 4, 4, 3, 3, 0, 1, 1, B.S4TF_F32, 0, 0)                    # stride 0
    assert L.s4tf_conv2d_fwd(ctypes.byref(bad), 16, 16, None, 16, None, 0, None) == -2
    bad = B.ConvDesc(1, 8, 8, 4, 4, 3, 3, 1, 1, 2, B.S4TF_F32, 0, 0)                    # 1 < groups < c
    assert L.s4tf_conv2d_fwd(ctypes.byref(bad), 16, 16, None, 16, None, 0, None) == -4
    bad = B.ConvDesc(1, 8, 8, 4, 4, 5, 5, 1, 2, 4, B.S4TF_F32, 0, 0)                    # depthwise, filter above 3x3
    assert L.s4tf_conv2d_fwd(ctypes.byref(bad), 16, 16, None, 16, None, 0, None) == -4
    assert "3x3" in B.last_error()
    bad = B.ConvDesc(1, 8, 8, 4, 4, 3, 3, 1, 1, 1, 7, 0, 0)                             # dtype
    assert L.s4tf_conv2d_fwd(ctypes.byref(bad), 16, 16, None, 16, None, 0, None) == -3
    bad = B.ConvDesc(1, 2, 2, 4, 4, 5, 5, 1, 0, 1, B.S4TF_F32, 0, 0)                    # filter > input
    assert L.s4tf_conv2d_fwd(ctypes.byref(bad), 16, 16, None, 16, None, 0, None) == -2
    # vjp with an activation needs y, and a workspace
    da = B.ConvDesc(4, 8, 8, 4, 4, 3, 3, 1, 1, 1, B.S4TF_F32, 1, 0)
    assert L.s4tf_conv2d_vjp(ctypes.byref(da), 16, 16, None, 16, None, 16, None, None, 0, None) == -1
    need = B.s4tf_conv2d_vjp_workspace_bytes(da)
    assert need > 0
    assert L.s4tf_conv2d_vjp(ctypes.byref(da), 16, 16, 16, 16, None, 16, None, 16, need - 1, None) == -5
    bn = B.BnDesc(2, 4, 4, 8, 1e-5, 1, B.S4TF_F32, 0)
    assert L.s4tf_bn_relu_fwd(ctypes.byref(bn), 16, None, 16, 16, 16, 16, 16, None, 0, None) == -5
    assert L.s4tf_sgd_momentum(0, None, None, None, None, 0.1, 0.9, None) == 0           # empty update is a no-op
    assert L.s4tf_sgd_momentum(4, None, 16, 16, None, 0.1, 0.9, None) == -1


def test_bad_networks_are_rejected():
    net = nets.tiny_block()
    # head not last
    broken = dict(net, ops=net["ops"][::-1])
    desc, keep = B.make_net_desc(broken)
    assert B.s4tf_net_param_count(desc) == 0 and B.last_error()
    # dangling tensor: a conv whose output nobody consumes
    ops = list(net["ops"])
    ops.insert(1, dict(ops[0], **{"in": 0}))
    ops[2] = dict(ops[2], **{"in": 1})
    ops[3] = dict(ops[3], **{"in": 3})
    desc, keep = B.make_net_desc(dict(net, ops=ops))
    assert B.s4tf_net_param_count(desc) == 0 and "consumer" in B.last_error()
    # residual of a different shape
    r = nets.resnet56(batch=2, blocks_per_stage=1, hw=8)
    ops = [dict(o) for o in r["ops"]]
    for o in ops:
        if o["kind"] == "bn" and o["res"] >= 0:
            o["res"] = 0
            break
    desc, keep = B.make_net_desc(dict(r, ops=ops))
    assert B.s4tf_net_param_count(desc) == 0 and "residual" in B.last_error()
    # params.count mismatch is caught before anything runs
    desc, keep = B.make_net_desc(net)
    p = B.Params(16, 16, 16, None, 3)
    b = B.Batch(16, 16, 16, 16, 1 << 30, None)
    assert B.lib().s4tf_train_step(ctypes.byref(desc), ctypes.byref(p), ctypes.byref(b), 0.1) == -2


def test_planned_networks_and_the_plan_cache():
    """s4tf_net_create plans a net once (Section 3.4's cache of compiled traces, keyed by a hash, is the
    model): equal descriptors hash alike, different ones differently; the schedule is a flat list whose
    length grows with the net; whatever makes a net impossible is reported at creation, before any launch;
    argument errors of a step on a plan are those of the descriptor form."""
    handles = {}
    for name in ("tiny", "lenet5", "resnet56", "resnet50", "mobilenetv2"):
        net = nets.CONFIGS[name]()
        desc, keep = B.make_net_desc(net)
        h = B.s4tf_net_create(desc)
        handles[name] = h
        assert h and B.s4tf_net_schedule_length(h) >= len([o for o in net["ops"] if o["kind"] != "flatten"])
        desc2, keep2 = B.make_net_desc(nets.CONFIGS[name]())     # an equal descriptor in other memory
        h2 = B.s4tf_net_create(desc2)
        assert h2 != h and B.s4tf_net_hash(h2) == B.s4tf_net_hash(h)
        assert B.s4tf_net_schedule_length(h2) == B.s4tf_net_schedule_length(h)
        B.s4tf_net_destroy(h2)
    assert len({B.s4tf_net_hash(h) for h in handles.values()}) == len(handles)
    other, keep = B.make_net_desc(nets.resnet56(batch=64))
    h3 = B.s4tf_net_create(other)
    assert B.s4tf_net_hash(h3) != B.s4tf_net_hash(handles["resnet56"])
    B.s4tf_net_destroy(h3)
    # the two small nets run on the caller's stream alone (no stream operations in their schedules):
    # conv, bn, head, bn pullback, filter gradient, optimizer = 6 commands
    assert B.s4tf_net_schedule_length(handles["tiny"]) == 6
    # a step on a plan validates its arguments like the descriptor form
    p = B.Params(16, 16, 16, None, 3)
    b = B.Batch(16, 16, 16, 16, 1 << 30, None)
    assert B.lib().s4tf_net_train_step(handles["tiny"], ctypes.byref(p), ctypes.byref(b), 0.1) == -2
    assert "params.count" in B.last_error()
    assert B.lib().s4tf_net_train_step(None, ctypes.byref(p), ctypes.byref(b), 0.1) == -1
    for h in handles.values():
        B.s4tf_net_destroy(h)
    B.s4tf_net_destroy(None)
    # impossible nets fail at creation
    net = nets.tiny_block()
    desc, keep = B.make_net_desc(dict(net, ops=net["ops"][::-1]))
    with pytest.raises(B.S4tfError):
        B.s4tf_net_create(desc)
    out = ctypes.c_void_p(123)
    assert B.lib().s4tf_net_create(None, ctypes.byref(out)) == -1 and out.value is None


def test_descriptor_calls_reuse_their_plan():
    """The descriptor form plans on first sight and looks the plan up afterwards: a query on a net of over a
    hundred ops costs microseconds once planned, and more plans than the cache holds are simply re-made."""
    import time
    net = nets.resnet50()
    desc, keep = B.make_net_desc(net)
    want = B.s4tf_train_step_workspace_bytes(desc)
    t0 = time.perf_counter()
    for _ in range(200):
        assert B.lib().s4tf_train_step_workspace_bytes(ctypes.byref(desc)) == want
    assert (time.perf_counter() - t0) / 200 < 2e-4
    for batch in range(1, 40):   # 39 different nets push the first plan out of the 32-entry cache
        d, k = B.make_net_desc(nets.lenet5(batch=batch))
        assert B.s4tf_net_param_count(d) == 61720   # 61 706 parameters, each tensor padded to a multiple of 8
    assert B.s4tf_train_step_workspace_bytes(desc) == want


def test_new_entry_points_reject_bad_arguments_on_the_host():
    L = B.lib()
    g = B.GatherDesc(10, 4, 3, B.S4TF_F32)
    assert L.s4tf_gather_rows_fwd(ctypes.byref(g), None, 16, 16, None) == -1
    assert L.s4tf_gather_rows_vjp(ctypes.byref(g), 16, 16, 8, None) == -7              # misaligned dx
    assert L.s4tf_gather_rows_fwd(ctypes.byref(B.GatherDesc(0, 4, 3, B.S4TF_F32)), 16, 16, 16, None) == -2
    assert L.s4tf_gather_rows_fwd(ctypes.byref(B.GatherDesc(10, 4, 0, B.S4TF_F32)), None, None, None, None) == 0   # nothing to gather
    assert L.s4tf_gather_rows_fwd(ctypes.byref(B.GatherDesc(10, 4, 3, 9)), 16, 16, 16, None) == -3
    assert L.s4tf_gather_rows_fwd(ctypes.byref(B.GatherDesc(1 << 20, 1 << 12, 3, B.S4TF_F32)), 16, 16, 16, None) == -2  # 2^32 elements
    bn = B.BnDesc(2, 4, 4, 8, 1e-5, 1, B.S4TF_F32, 0, 0)
    assert L.s4tf_bn_inference_fwd(ctypes.byref(bn), 16, None, 16, 16, None, 16, 16, None) == -1      # running_mean missing
    assert L.s4tf_bn_update_running(0, 10, 0.1, 1e-5, 16, 16, 16, 16, None) == -2
    assert L.s4tf_bn_update_running(8, 10, 1.5, 1e-5, 16, 16, 16, 16, None) == -2                     # momentum out of [0, 1]
    cd = B.ConvDesc(1, 8, 8, 4, 4, 3, 3, 1, 1, 1, B.S4TF_F32, 0, 0)
    assert L.s4tf_bn_fold_into_conv(ctypes.byref(cd), 16, None, 16, 16, 16, 16, -1.0, 16, 16, None) == -2   # eps < 0
    assert L.s4tf_bn_fold_into_conv(ctypes.byref(cd), 16, None, 16, 16, 16, 16, 1e-5, None, 16, None) == -1
    assert L.s4tf_round_to_bf16(0, None, None, None) == 0
    assert L.s4tf_round_to_bf16(4, None, 16, None) == -1
    # tensors beyond the kernels' 32-bit element indices are refused, not wrapped
    huge = B.ConvDesc(1 << 10, 1 << 10, 1 << 10, 4, 4, 1, 1, 1, 0, 1, B.S4TF_F32, 0, 0)
    assert L.s4tf_conv2d_fwd(ctypes.byref(huge), 16, 16, None, 16, None, 0, None) == -2 and "2^31" in B.last_error()
    # the allocation-free BatchNorm forward: capacity query needs no device, the refusal comes before any launch
    big = B.BnDesc(64, 56, 56, 512, 1e-5, 1, B.S4TF_BF16, 0, 0)
    cap, needed = B.s4tf_bn_relu_fwd_static_limit(big)
    assert cap == 1 << 20 and needed > cap
    assert L.s4tf_bn_relu_fwd_static(ctypes.byref(big), 16, None, 16, 16, 16, 16, 16, None) == -5


def test_seeded_random_descriptors_never_get_past_the_host_checks():
    """2000 convolution, BatchNorm and pool descriptors with fields drawn from valid and invalid values, data
    pointers NULL: every call must come back with an error status (a bad descriptor's own, else NULL) and an
    error text, every workspace query with a size, and nothing may crash.  No device is touched."""
    L = B.lib()
    rng = np.random.default_rng(77)
    vals = [-3, 0, 1, 2, 3, 4, 5, 7, 8, 16, 24, 64, 224, 1 << 12, 1 << 20, (1 << 31) - 1]
    small = [-1, 0, 1, 2, 3, 5, 7]
    seen = set()
    for _ in range(2000):
        pick = lambda v: int(rng.choice(v))
        d = B.ConvDesc(pick(vals), pick(vals), pick(vals), pick(vals), pick(vals), pick(small), pick(small), pick(small),
                       pick(small), pick([0, 1, 2, 4, 8, 16, 64]), pick([0, 1, 2, -1]), pick([0, 1, 2, 3]), pick([0, 1]))
        rc = L.s4tf_conv2d_fwd(ctypes.byref(d), None, None, None, None, None, 0, None)
        assert rc in (-1, -2, -3, -4), rc
        assert B.last_error()
        seen.add(rc)
        rc = L.s4tf_conv2d_vjp(ctypes.byref(d), None, None, None, None, None, None, None, None, 0, None)
        assert rc in (-1, -2, -3, -4), rc
        assert B.s4tf_conv2d_vjp_workspace_bytes(d) >= 0
        assert B.s4tf_conv2d_fwd_workspace_bytes(d) >= 0
        bd = B.BnDesc(pick(vals), pick(vals), pick(vals), pick(vals), float(rng.choice([-1.0, 0.0, 1e-5, float("nan")])),
                      pick([0, 1, 2, 3]), pick([0, 1, 2]), pick([0, 1]))
        rc = L.s4tf_bn_relu_fwd(ctypes.byref(bd), None, None, None, None, None, None, None, None, 0, None)
        assert rc in (-1, -2, -3, -4), rc
        assert int(L.s4tf_bn_relu_workspace_bytes(ctypes.byref(bd))) >= 0
        pd = B.PoolDesc(pick(vals), pick(vals), pick(vals), pick(vals), pick([0, 1, 2, -1]), pick([0, 1, 2]), pick([0, 1]))
        rc = L.s4tf_pool2d_fwd(ctypes.byref(pd), None, None, None)
        assert rc in (-1, -2, -3, -4), rc
    assert seen == {-1, -2, -3, -4}, seen   # valid descriptors (NULL pointers) and each kind of bad one occurred


def test_seeded_random_networks_are_planned_or_refused_without_a_crash():
    """3000 op lists with kinds, tensor references and sizes drawn at random (mostly nonsense, some valid by
    construction: a mutated valid net).  Planning must either give a handle whose queries are sane or refuse with an
    error text; no crash, no handle for a net whose head is not its last op.  No device is touched."""
    L = B.lib()
    rng = np.random.default_rng(4242)
    base = nets.resnet56(batch=2, blocks_per_stage=1, hw=8)
    planned = refused = 0
    for it in range(3000):
        if it % 3 == 0:    # a valid net with a few fields mutated
            ops = [dict(o) for o in base["ops"]]
            for _ in range(int(rng.integers(1, 4))):
                o = ops[int(rng.integers(len(ops)))]
                key = str(rng.choice(["in", "k", "r", "stride", "pad", "res", "groups"]))
                if key in o:
                    o[key] = int(rng.choice([-2, -1, 0, 1, 2, 3, 5, 7, 16, 1 << 20]))
                    if key == "r":
                        o["s"] = o[key]
            desc, keep = B.make_net_desc(dict(base, ops=ops))
        else:              # raw op records
            n_ops = int(rng.integers(1, 12))
            ops = (B.Op * n_ops)()
            for i, o in enumerate(ops):
                o.kind = int(rng.integers(-1, 8))
                o.in_ = int(rng.integers(-2, n_ops + 2))
                o.res = int(rng.integers(-2, n_ops + 2))
                o.k = int(rng.choice([-1, 0, 1, 4, 10, 16, 1 << 24]))
                o.r = o.s = int(rng.choice([-1, 0, 1, 3, 5, 9]))
                o.stride = int(rng.choice([-1, 0, 1, 2, 3]))
                o.pad = int(rng.choice([-1, 0, 1, 2, 100]))
                o.groups = int(rng.choice([-1, 0, 1, 2, 4, 16]))
                o.has_bias = int(rng.integers(0, 2))
                o.act = int(rng.integers(-1, 4))
                o.eps = float(rng.choice([-1.0, 0.0, 1e-5]))
            if rng.random() < 0.5:
                ops[n_ops - 1].kind = B.OP_HEAD
            desc = B.NetDesc(int(rng.choice([0, 1, 2, 8])), int(rng.choice([0, 1, 8, 32])), int(rng.choice([1, 8, 32])),
                             int(rng.choice([0, 1, 3, 4])), int(rng.choice([0, 1, 5])), n_ops, ops, 0.9)
            keep = ops
        out = ctypes.c_void_p()
        rc = L.s4tf_net_create(ctypes.byref(desc), ctypes.byref(out))
        if rc == 0:
            planned += 1
            assert out.value
            assert desc.ops[desc.n_ops - 1].kind == B.OP_HEAD
            assert B.s4tf_net_param_count(desc) > 0
            assert B.s4tf_train_step_workspace_bytes(desc) > 0
            L.s4tf_net_destroy(out)
        else:
            refused += 1
            assert rc < 0 and B.last_error()
            assert not out.value
    assert planned >= 50 and refused >= 1000, (planned, refused)
