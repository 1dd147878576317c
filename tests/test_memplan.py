"""Memory planning (Relax, Sec. 4.3, Algorithm 3): pins of the plain reference planner in oracle/memplan.py, and the
library's plan of the layer workspace (relax_workspace_plan, host-only) against it."""
import itertools

import pytest

from oracle import memplan
from paper_2311_02103_amd import binding as rx


# ------------------------------------------------------------------------------------------------ pins of the reference
def chain(sizes):
    """t0 = f(x); t1 = f(t0); ...: every operation reads the previous tensor and writes the next."""
    prog = []
    for i, s in enumerate(sizes):
        prog.append(("alloc", "t%d" % i, s))
        prog.append(("call", "op%d" % i, (["t%d" % (i - 1)] if i else []) + ["t%d" % i]))
    return prog


def test_four_intermediates_of_equal_symbolic_shape_share_two_storages():
    """The example of the paper's memory-planning figure: four intermediate tensors, individually allocated before
    planning, live in two storage chunks afterwards."""
    prog = chain([("rows", 16)] * 4)
    for rule in ("equal", "fits"):                                 # the paper's rule, and the extension: the example needs only equality
        storage_of, sizes = memplan.plan(prog, outputs=["t3"], rule=rule)
        assert len(sizes) == 2
        assert [storage_of["t%d" % i] for i in range(4)] == [0, 1, 0, 1]
        assert sizes == [("rows", 16), ("rows", 16)]


def test_equality_rule_reuses_only_the_same_expression():
    """Sec. 4.3 reuses a storage when the two symbolic sizes are proven equal: n*8 and n*4 are different expressions, so the
    paper's rule opens a new storage where the "provably fits" extension parks the smaller tensor in the larger one."""
    prog = chain([("rows", 8), ("rows", 8), ("rows", 4), ("rows", 8)])
    eq_of, eq_sizes = memplan.plan(prog, outputs=["t3"], rule="equal")
    assert eq_sizes == [("rows", 8), ("rows", 8), ("rows", 4)]
    assert eq_of == {"t0": 0, "t1": 1, "t2": 2, "t3": 0}           # t2 (4n) gets its own storage; t3 (8n) reuses t0's, free since t1
    fit_of, fit_sizes = memplan.plan(prog, outputs=["t3"], rule="fits")
    assert fit_sizes == [("rows", 8), ("rows", 8)] and fit_of == {"t0": 0, "t1": 1, "t2": 0, "t3": 1}
    # opaque expressions: only the same expression, under both rules
    prog = chain([("opaque", 1), ("opaque", 2), ("opaque", 1), ("opaque", 2)])
    for rule in ("equal", "fits"):
        of, sizes = memplan.plan(prog, outputs=["t3"], rule=rule)
        assert sizes == [("opaque", 1), ("opaque", 2)] and of == {"t0": 0, "t1": 1, "t2": 0, "t3": 1}
    # neither rule dominates the other in bytes: the walk is greedy, and parking a small tensor in a big free storage (which
    # only the extension may do) can force a new big storage later
    sizes_ = [("rows", 9), ("rows", 3), ("rows", 3), ("rows", 9), ("rows", 1)]
    pe = memplan.planned_bytes(memplan.plan(chain(sizes_), ["t4"], rule="equal")[1], 1000, {})
    pf = memplan.planned_bytes(memplan.plan(chain(sizes_), ["t4"], rule="fits")[1], 1000, {})
    assert (pe, pf) == (9216 + 3072 + 3072 + 1024, 9216 + 3072 + 9216)      # storages {9n, 3n, 3n, 1n} against {9n, 3n, 9n} at n = 1000


def test_planned_bytes_closed_forms():
    """The byte count of a plan is the sum of its storages, each evaluated at the symbols' values and rounded up to the
    alignment: written out by hand here."""
    assert memplan.evaluate(("rows", 100), 3, {}) == 300
    assert memplan.evaluate(("opaque", 7), 3, {7: 1000}) == 1000
    assert memplan.planned_bytes([("rows", 100), ("opaque", 1)], 3, {1: 1000}) == 512 + 1024            # 300 -> 512, 1000 -> 1024
    assert memplan.planned_bytes([("rows", 256)], 1, {}) == 256                                          # exact multiples stay
    assert memplan.planned_bytes([("rows", 256)], 2, {}) == 512
    assert memplan.planned_bytes([("rows", 1)], 257, {}) == 512
    assert memplan.planned_bytes([("rows", 1), ("rows", 1)], 1, {}, align=64) == 128
    assert memplan.planned_bytes([], 5, {}) == 0
    # the four equal intermediates of the figure at n = 10 rows of 16 bytes: two storages of 160 -> 256 bytes each
    assert memplan.planned_bytes(memplan.plan(chain([("rows", 16)] * 4), ["t3"], rule="equal")[1], 10, {}) == 512


def test_symbolically_different_sizes_are_not_reused_unless_they_provably_fit():
    # n*8 then n*4: the smaller fits the freed larger one; the other way round it does not
    s1, _ = memplan.plan(chain([("rows", 8), ("rows", 8), ("rows", 4)]), outputs=["t2"])
    assert s1["t2"] == s1["t0"]
    s2, sizes2 = memplan.plan(chain([("rows", 4), ("rows", 4), ("rows", 8)]), outputs=["t2"])
    assert len(sizes2) == 3 and len({s2["t0"], s2["t1"], s2["t2"]}) == 3
    # an opaque expression is reused only by the same expression, never by a rows-sized tensor or another expression
    s3, sizes3 = memplan.plan(chain([("opaque", 1), ("opaque", 1), ("opaque", 2), ("rows", 1), ("opaque", 1)]), outputs=["t4"])
    assert s3["t4"] == s3["t0"] and s3["t2"] not in (s3["t0"], s3["t1"]) and s3["t3"] not in (s3["t0"], s3["t1"], s3["t2"])


def test_best_fit_takes_the_smallest_free_storage_that_holds_the_request():
    prog = [("alloc", "a", ("rows", 10)), ("alloc", "b", ("rows", 6)), ("alloc", "c", ("rows", 8)), ("call", "f", ["a", "b", "c"]),
            ("alloc", "d", ("rows", 7)), ("call", "g", ["d"])]
    storage_of, _ = memplan.plan(prog, outputs=["d"])
    assert storage_of["d"] == storage_of["c"]                      # 8 n is the smallest of the free {10 n, 6 n, 8 n} that holds 7 n


def live_ranges(prog, outputs):
    last = memplan.liveness(prog, outputs)
    first = {op[1]: i for i, op in enumerate(prog) if op[0] == "alloc"}
    return {t: (first[t], last[t]) for t in first}


def overlapping(r1, r2):
    return r1[0] <= r2[1] and r2[0] <= r1[1]


def min_storages_brute_force(prog, outputs):
    """Fewest storages of ANY valid assignment (tensors that are live together never share; a tensor fits the storage's
    first tenant or the first tenant fits... every tenant must fit the largest one): exhaustive over set partitions."""
    rng = live_ranges(prog, outputs)
    size = {op[1]: op[2] for op in prog if op[0] == "alloc"}
    names = list(rng)
    best = len(names)
    for labels in itertools.product(range(len(names)), repeat=len(names)):
        if any(labels[i] > max(labels[:i], default=-1) + 1 for i in range(len(names))):
            continue                                               # canonical labelling only
        groups = {}
        for nme, g in zip(names, labels):
            groups.setdefault(g, []).append(nme)
        ok = True
        for members in groups.values():
            for a, b in itertools.combinations(members, 2):
                if overlapping(rng[a], rng[b]):
                    ok = False
            # one storage size must provably hold every member: the member that all others fit into
            if not any(all(memplan.provably_fits(size[m], size[h]) for m in members) for h in members):
                ok = False
        if ok:
            best = min(best, len(groups))
    return best


@pytest.mark.parametrize("sizes,optimal", [([("rows", 4)] * 5, True),
                                           ([("rows", 4), ("rows", 4), ("opaque", 1), ("rows", 4), ("opaque", 1)], True),
                                           # the walk is greedy in program order: here it parks a small tensor in the big free
                                           # storage and has to open a third one, where two would do
                                           ([("rows", 9), ("rows", 3), ("rows", 3), ("rows", 9), ("rows", 1)], False)])
def test_chains_against_the_fewest_storages_any_assignment_can_reach(sizes, optimal):
    prog = chain(sizes)
    out = ["t%d" % (len(sizes) - 1)]
    storage_of, storage_sizes = memplan.plan(prog, outputs=out)
    fewest = min_storages_brute_force(prog, out)
    assert len(storage_sizes) == fewest if optimal else len(storage_sizes) == fewest + 1
    rng = live_ranges(prog, out)
    size = {op[1]: op[2] for op in prog if op[0] == "alloc"}
    for a, b in itertools.combinations(rng, 2):                   # tensors that are live together never share a storage
        if overlapping(rng[a], rng[b]):
            assert storage_of[a] != storage_of[b]
    for t, s in storage_of.items():                               # and every tensor provably fits its storage
        assert memplan.provably_fits(size[t], storage_sizes[s])


# ------------------------------------------------------------------------------------------------ the library's plan
def layer_program(hidden, n_heads, n_kv_heads, head_dim, ffn):
    """The layer as its sequence of destination-passing operations (norm + QKV + rotary + append, attention, output
    projection + residual, gate/up + SwiGLU, down + residual; the second norm
    is an operation of its own), with the sizes of its intermediates in bytes per row, written out independently of
    the library: xn fp16 [n,H]; qkv fp16 [n,(h+2g)d]; attention output fp16 [n,hd]; x1 fp32 [n,H]; act fp16 [n,F]; the
    lifted workspaces of the few-row matmul (one expression, requested around each matmul) and of split-L attention."""
    H, hd, qkvw = hidden, n_heads * head_dim, (n_heads + 2 * n_kv_heads) * head_dim
    MM, PART = 1, 2
    prog = [
        ("alloc", "xn", ("rows", 2 * H)),
        ("alloc", "qkv", ("rows", 2 * qkvw)), ("alloc", "matmul_ws.qkv", ("opaque", MM)),
        ("call", "norm+qkv+rope+append", ["xn", "matmul_ws.qkv", "qkv"]),
        ("alloc", "attn_partials", ("opaque", PART)), ("alloc", "attn_out", ("rows", 2 * hd)),
        ("call", "attention", ["qkv", "attn_partials", "attn_out"]),
        ("alloc", "x1", ("rows", 4 * H)), ("alloc", "matmul_ws.o", ("opaque", MM)),
        ("call", "o_proj+residual", ["attn_out", "attn_partials", "matmul_ws.o", "x1"]),      # the folded merge reads the partials here
        ("call", "norm2", ["x1", "xn"]),
        ("alloc", "act", ("rows", 2 * ffn)), ("alloc", "matmul_ws.gate_up", ("opaque", MM)),
        ("call", "gate_up+swiglu", ["xn", "matmul_ws.gate_up", "act"]),
        ("alloc", "matmul_ws.down", ("opaque", MM)),
        ("call", "down+residual", ["act", "x1", "matmul_ws.down", "xn"]),                    # also leaves the next layer's xn
    ]
    return prog, ["xn"]


SHAPES = {"7B": dict(hidden=4096, n_heads=32, n_kv_heads=32, head_dim=128, ffn=11008),
          "70B": dict(hidden=8192, n_heads=64, n_kv_heads=8, head_dim=128, ffn=28672),
          "tiny": dict(hidden=256, n_heads=4, n_kv_heads=4, head_dim=64, ffn=688)}


@pytest.mark.parametrize("rule", ["fits", "equal"])
@pytest.mark.parametrize("shape", list(SHAPES))
@pytest.mark.parametrize("n,L,B", [(1, 1, 1), (1, 4096, 1), (16, 8000, 16), (64, 300, 64), (128, 128, 1), (512, 512, 2), (2048, 2048, 1)])
def test_library_plan_equals_the_reference_plan(shape, n, L, B, rule):
    sh = SHAPES[shape]
    cap = 8192
    dims = rx.make_dims(sh["hidden"], sh["n_heads"], sh["n_kv_heads"], sh["head_dim"], sh["ffn"], cap, max(B, 1))
    if rule == "fits":                                            # the rule the workspace is laid out with: the plain query reports it
        rc, entries, planned, unplanned = rx.relax_workspace_plan(dims, n, L, B)
        assert (rc, entries, planned, unplanned) == rx.relax_workspace_plan(dims, n, L, B, rule=0)
    else:                                                         # the paper's rule: equal expressions only
        rc, entries, planned, unplanned = rx.relax_workspace_plan(dims, n, L, B, rule=1)
    assert rc == 0
    by_name = {e["name"]: e for e in entries}
    prog, outputs = layer_program(**sh)
    storage_of, storage_sizes = memplan.plan(prog, outputs, rule=rule)
    assert set(by_name) == set(storage_of)
    # same sharing structure (storage numbers are arbitrary labels on both sides: compare the partition of the tensors)
    part_lib, part_ref = {}, {}
    for t in storage_of:
        part_lib.setdefault(by_name[t]["storage"], set()).add(t)
        part_ref.setdefault(storage_of[t], set()).add(t)
    assert sorted(map(sorted, part_lib.values())) == sorted(map(sorted, part_ref.values()))
    # sizes: the rows-sized tensors are the bytes written out above; the two opaque expressions are workload parameters of the
    # library (functions of n, L, B that its kernels define), taken as given -- they are inputs of the planner, not results
    sizes = {op[1]: op[2] for op in prog if op[0] == "alloc"}
    opaque = {}
    for t, sz in sizes.items():
        if sz[0] == "rows":
            assert by_name[t]["bytes"] == sz[1] * n, t
        else:
            opaque.setdefault(sz[1], by_name[t]["bytes"])
            assert by_name[t]["bytes"] == opaque[sz[1]], "one expression, one value"
    assert planned == memplan.planned_bytes(storage_sizes, n, opaque)
    assert unplanned == sum((by_name[t]["bytes"] + 255) // 256 * 256 for t in sizes)
    # validity from the reference's liveness: tensors that are live together do not overlap in the workspace
    rng = live_ranges(prog, outputs)
    for a, b in itertools.combinations(rng, 2):
        if overlapping(rng[a], rng[b]):
            ea, eb = by_name[a], by_name[b]
            assert ea["offset"] + ea["bytes"] <= eb["offset"] or eb["offset"] + eb["bytes"] <= ea["offset"], (a, b)
    for e in entries:
        assert e["offset"] % 256 == 0 and e["bytes"] <= e["storage_bytes"]
    if rule == "fits":
        assert rx.relax_workspace_bytes(dims, n, L, B) == max(e["offset"] + (e["storage_bytes"] + 255) // 256 * 256 for e in entries)


def test_plan_at_upper_bounds_covers_every_smaller_call():
    """Static planning from upper bounds (Sec. 4.3): every storage grows with the symbols, so no tensor of a smaller call
    reaches past the workspace sized at (n_max, L_max, B_max)."""
    sh = SHAPES["7B"]
    dims = rx.make_dims(sh["hidden"], sh["n_heads"], sh["n_kv_heads"], sh["head_dim"], sh["ffn"], 4096, 64)
    total = rx.relax_workspace_bytes(dims, 2048, 4096, 64)
    for n, L, B in [(1, 1, 1), (1, 4096, 1), (7, 4096, 7), (64, 4096, 64), (129, 200, 3), (2048, 2048, 1), (2048, 4096, 64)]:
        rc, entries, _, _ = rx.relax_workspace_plan(dims, n, L, B)
        assert rc == 0
        assert max(e["offset"] + e["bytes"] for e in entries) <= total
        assert rx.relax_workspace_bytes(dims, n, L, B) <= total


def test_plan_query_errors():
    dims = rx.make_dims(256, 4, 4, 64, 688, 64, 1)
    assert rx.relax_workspace_plan(None, 1, 1, 1)[0] == rx.ERR_NULL
    assert rx.relax_workspace_plan(dims, 0, 1, 1)[0] == rx.ERR_SHAPE
    assert rx.relax_workspace_plan(dims, 1, 1, 1, capacity=3)[0] == rx.ERR_WORKSPACE
    assert rx.relax_workspace_plan(dims, 1, 1, 1, rule=2)[0] == rx.ERR_UNSUPPORTED
    assert rx.relax_workspace_plan(dims, 1, 1, 1, rule=1)[0] == 0
