"""The C-ABI library loads and exports every symbol include/pb.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

import pb_workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "pb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pb_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    from paper_2003_11666_amd import binding as B
    if not os.path.exists(B.lib_path()):
        from paper_2003_11666_amd import build
        build.build(verbose=False)
    lib = B.load_library()
    names = _declared()
    assert "pb_init" in names and "pb_tick" in names and "pb_read_weights" in names \
        and "pb_loss_history" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_descriptor_validation_on_host():
    from paper_2003_11666_amd import binding as B
    lib = B.load_library()
    for name in ("mlp", "vgg11", "resnet20", "wide", "resnet50", "resnet50_64", "tiny_bottleneck"):
        d, keep = B.marshal_net(W.config(name))
        assert lib.pb_arena_bytes(ctypes.byref(d), None) > 0, name
    # the pipeline's own delays, larger ones (deeper weight-version rings, more memory) and smaller ones
    # (sample-indexed form) are all accepted; negative ones are refused
    net = W.config("tiny_resnet")
    S = len(net["stages"])
    d, keep = B.marshal_net(net)
    nat = (ctypes.c_int32 * S)(*[2 * (S - 1 - s) for s in range(S)])
    assert lib.pb_arena_bytes(ctypes.byref(d), nat) > 0
    zero = (ctypes.c_int32 * S)(*([0] * S))
    assert lib.pb_arena_bytes(ctypes.byref(d), zero) > 0
    neg = (ctypes.c_int32 * S)(*([0] * (S - 1) + [-1]))
    assert lib.pb_arena_bytes(ctypes.byref(d), neg) == 0
    assert b"negative" in lib.pb_last_error()
    more = (ctypes.c_int32 * S)(*[2 * (S - 1 - s) + 3 for s in range(S)])
    assert lib.pb_arena_bytes(ctypes.byref(d), more) > lib.pb_arena_bytes(ctypes.byref(d), nat)
    # broken descriptor: loss op missing
    bad = dict(net)
    bad["stages"] = [list(st) for st in net["stages"]]
    bad["stages"][-1] = bad["stages"][-1][:-1]
    d, keep = B.marshal_net(bad)
    assert lib.pb_arena_bytes(ctypes.byref(d), None) == 0


def test_hyperparameter_scaling_is_host_arithmetic():
    """pb_scale_hyperparameters (Eq. hpscale) touches no device: checked here against the oracle's
    routine and against the two invariants the appendix states."""
    from paper_2003_11666_amd import binding as B
    from oracle import pb_oracle as O
    lib = B.load_library()
    for lr_r, m_r, n_r, n in [(0.1, 0.9, 128, 1), (0.1, 0.9, 32, 1), (0.05, 0.95, 64, 8)]:
        lr, m = B.scale_hyperparameters(lr_r, m_r, n_r, n)
        lo, mo = O.scale_hyperparameters(lr_r, m_r, n_r, n)
        assert abs(lr - lo) <= 1e-6 * lo and abs(m - mo) <= 1e-7
    out = ctypes.c_float()
    assert lib.pb_scale_hyperparameters(0.1, 0.9, 0, 1, ctypes.byref(out), ctypes.byref(out)) < 0
    assert lib.pb_scale_hyperparameters(0.1, 1.5, 8, 1, ctypes.byref(out), ctypes.byref(out)) < 0
    assert lib.pb_scale_hyperparameters(0.1, 0.9, 8, 1, None, ctypes.byref(out)) < 0


def _plan(name):
    from paper_2003_11666_amd import binding
    rows = []
    for line in binding.plan_summary(W.config(name)).splitlines():
        m = re.match(r"stage\s+(\d+) phase (\d+) (\S+)\s+tiles\s+(\d+)", line)
        assert m, line
        rows.append((int(m.group(1)), int(m.group(2)), m.group(3), int(m.group(4)), line))
    return rows


def test_resnet20_plan_two_phases_split_weight_gradients_short_steps_first():
    """Host-side planning of the headline configuration: two launches per tick; the weight
    gradients of the 32x32 layers are split over workgroups; a phase begins with its short steps."""
    rows = _plan("resnet20")
    assert {r[1] for r in rows} == {0, 1}
    split = [r for r in rows if "gm3" in r[4] and "C16x32x32 K16x32x32 k3" in r[4]]
    assert len(split) == 6
    for r in split:
        m = re.search(r"chunks (\d+)/(\d+)", r[4])
        assert int(m.group(2)) >= 4 and int(m.group(1)) >= int(m.group(2))
    phase0 = [r for r in rows if r[1] == 0]
    kinds = [r[2] for r in phase0]
    first_gemm = kinds.index("gemm")
    assert set(kinds[:first_gemm]) <= {"ingest", "copy", "gn_stats", "head"}
    assert "gn_stats" not in kinds[first_gemm:] and "ingest" not in kinds[first_gemm:]
    # GroupNorm statistics of a layer of four groups: one workgroup
    assert all(r[3] == 1 for r in phase0 if r[2] == "gn_stats")


def test_throughput_plans_keep_every_tile_count_consistent():
    for name in ("vgg11", "wide"):
        for r in _plan(name):
            if r[2] != "gemm":
                continue
            m = re.search(r"chunks (\d+)/(\d+)", r[4])
            chunks, parts = int(m.group(1)), int(m.group(2))
            assert 1 <= parts <= chunks and r[3] % parts == 0, r[4]


def test_split_test_network_really_splits():
    """The small network the GPU tests use for the split weight-gradient reduction is planned that way."""
    rows = [r for r in _plan("split_resnet") if "gm3" in r[4]]
    parts = [int(re.search(r"chunks (\d+)/(\d+)", r[4]).group(2)) for r in rows]
    assert max(parts) >= 4



def test_planner_settings_struct_matches_the_header():
    """The binding's copy of pb_tuning has the header's fields, in the header's order."""
    from paper_2003_11666_amd import binding as B
    text = open(os.path.join(ROOT, "include", "pb.h")).read()
    body = re.search(r"typedef struct \{([^}]*)\} pb_tuning;", text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = []
    for decl in body.split(";"):
        decl = decl.strip()
        if decl:
            names += [n.strip() for n in decl.split(None, 1)[1].split(",")]
    assert names == [f[0] for f in B._Tuning._fields_]
