"""Host-side logic of the library, through the C ABI, against the oracle and the paper's examples (no GPU)."""
import ctypes as C
import os
import random
import re

import numpy as np
import pytest

from paper_2111_14255_amd import binding as B, api
from oracle import schedule as S, fold as ofold, ops as oops
from synth import zoo, weights

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
I32 = C.c_int32


def arr(vals):
    return (I32 * max(1, len(vals)))(*vals)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "mtsched.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(mt_[a-z0-9_]+)\s*\(", hdr)) - {"mt_cost_fn"}
    declared -= {"mt_share_cost_fn"}
    assert declared == set(B.SIGNATURES), declared ^ set(B.SIGNATURES)
    lib = B.load()
    for name in declared:
        assert getattr(lib, name) is not None


def lib_expand(lens, rho, n_stages):
    n = len(lens)
    flat = [v for r in rho for v in r]
    out = (I32 * (n_stages * n * 2))()
    rc = B.load().mt_expand_pointers(n, arr(lens), n_stages, arr(flat), out)
    if rc != 0:
        return rc
    return [[(out[(s * n + i) * 2], out[(s * n + i) * 2 + 1]) for i in range(n)] for s in range(n_stages)]


def test_expand_worked_examples():
    st = lib_expand([10], [[3, 5, 7]], 4)
    assert [list(range(b + 1, e + 1)) for (b, e), in st] == [[1, 2, 3], [4, 5], [6, 7], [8, 9, 10]]
    st = lib_expand([10, 4, 5], [[3, 5], [1, 2], [2, 2]], 3)
    assert st[0] == [(0, 3), (0, 1), (0, 2)] and st[1] == [(3, 5), (1, 2), (2, 2)]


def test_expand_matches_oracle_random():
    rng = random.Random(1)
    for _ in range(300):
        n, p = rng.randint(1, 8), rng.randint(0, 7)
        lens = [rng.randint(1, 150) for _ in range(n)]
        rho = [sorted(rng.randint(0, L) for _ in range(p)) for L in lens]
        assert lib_expand(lens, rho, p + 1) == [list(s) for s in S.expand(lens, rho)]


def test_expand_rejects_invalid():
    assert lib_expand([5], [[3, 2]], 3) == B.MT_ERR_INVALID_SCHEDULE
    assert b"non-decreasing" in B.load().mt_last_error()
    assert lib_expand([5], [[6]], 2) == B.MT_ERR_INVALID_SCHEDULE
    assert lib_expand([5], [[1] * 16], 17) == B.MT_ERR_INVALID_SCHEDULE


def lib_issue(stage, conc, order):
    n = len(stage)
    flat = [v for s in stage for v in s]
    total = sum(e - b for b, e in stage)
    out = (I32 * max(1, 3 * total))()
    cnt = I32()
    rc = B.load().mt_issue_order_of_stage(n, arr(flat), conc, order, out, C.byref(cnt))
    assert rc == 0
    return [(out[3 * k], out[3 * k + 1], out[3 * k + 2]) for k in range(cnt.value)]


def test_issue_order_examples_and_oracle():
    stage = [(0, 3), (0, 1), (0, 2)]
    assert [(s + 1, i + 1) for s, t, i in lib_issue(stage, 3, B.MT_ISSUE_BFS)] == [(1, 1), (2, 1), (3, 1), (1, 2), (3, 2), (1, 3)]
    assert [(s + 1, i + 1) for s, t, i in lib_issue(stage, 3, B.MT_ISSUE_DFS)] == [(1, 1), (1, 2), (1, 3), (2, 1), (3, 1), (3, 2)]
    rng = random.Random(2)
    for _ in range(300):
        n = rng.randint(1, 8)
        stage = []
        for _ in range(n):
            b = rng.randint(0, 20)
            stage.append((b, b + rng.choice([0, 0, 1, 2, 5, 9])))
        conc = rng.randint(1, n + 1)
        for order, name in ((B.MT_ISSUE_BFS, "bfs"), (B.MT_ISSUE_DFS, "dfs")):
            assert lib_issue(stage, conc, order) == S.issue_order(stage, conc, name)


def lib_search(lens, n_stages, rounds, cands, seed, algo, cost, seed_baselines=0):
    n, P = len(lens), n_stages - 1
    opts = B.mt_search_opts(algo, n_stages, rounds, cands, 1, 0, 0, 0, seed_baselines, 0, 0, 0, 0, 0, seed)
    cap = rounds * n * cands + 2
    best = (I32 * max(1, n * P))()
    bc = C.c_double()
    recp = (I32 * max(1, cap * n * P))()
    recc = (C.c_double * cap)()
    nrec = I32()

    def cb(ptr, _user):
        return cost([[ptr[i * P + j] for j in range(P)] for i in range(n)])

    fn = B.mt_cost_fn(cb)
    rc = B.load().mt_search_pointers(n, arr(lens), C.byref(opts), fn, None, best, C.byref(bc), recp, recc, cap, C.byref(nrec))
    assert rc == 0, B.load().mt_last_error()
    rho = [[best[i * P + j] for j in range(P)] for i in range(n)]
    recs = [([[recp[(k * n + i) * P + j] for j in range(P)] for i in range(n)], recc[k]) for k in range(nrec.value)]
    return rho, bc.value, recs


def _cost(target):
    return lambda rho: float(sum((a - b) ** 2 for r, t in zip(rho, target) for a, b in zip(r, t))) + 0.5


def test_coordinate_descent_matches_oracle():
    lens = [23, 21, 54]
    target = [[5, 11, 17], [3, 9, 20], [10, 30, 50]]
    for seed in (1, 7, 123456789):
        rho, c, recs = lib_search(lens, 4, 3, 4, seed, B.MT_SEARCH_COORDINATE, _cost(target))
        orho, oc, orecs = S.coordinate_descent(lens, 3, 3, 4, _cost(target), seed)
        assert recs == [(r, c2) for r, c2 in orecs]
        assert rho == orho and c == oc
        assert len(recs) == 3 * 3 * 4


def test_search_with_baseline_seeds_matches_oracle():
    lens = [23, 21, 54]
    target = [[23, 23, 23], [21, 21, 21], [50, 52, 54]]       # close to "everything in stage 1"
    for algo, fn in ((B.MT_SEARCH_COORDINATE, lambda: S.coordinate_descent(lens, 3, 2, 3, _cost(target), 5, seed_baselines=True)[:3]),
                     (B.MT_SEARCH_RANDOM, lambda: S.random_search(lens, 3, 2 * 3 * 3, _cost(target), 5, seed_baselines=True)[:3])):
        rho, c, recs = lib_search(lens, 4, 2, 3, 5, algo, _cost(target), seed_baselines=1)
        orho, oc, orecs = fn()
        assert recs == orecs and rho == orho and c == oc
        assert recs[0][0] == [[23] * 3, [21] * 3, [54] * 3] and recs[1][0] == S.even_split(lens, 3)


def test_random_search_matches_oracle():
    lens = [9, 12]
    target = [[2, 6], [4, 8]]
    rho, c, recs = lib_search(lens, 3, 10, 5, 99, B.MT_SEARCH_RANDOM, _cost(target))
    orho, oc, orecs, skipped = S.random_search(lens, 2, 10 * 2 * 5, _cost(target), 99)
    assert recs == orecs and rho == orho and c == oc and skipped > 0


def lib_playoff(lens, n_stages, recs, top_k, cost):
    n, P = len(lens), n_stages - 1
    flat = [v for rho, _ in recs for row in rho for v in row]
    costs = (C.c_double * max(1, len(recs)))(*[c for _, c in recs])
    best = (I32 * max(1, n * P))()
    bc = C.c_double()
    nev = I32()
    seen = []

    def cb(ptr, _user):
        rho = [[ptr[i * P + j] for j in range(P)] for i in range(n)]
        seen.append(rho)
        return cost(rho)

    fn = B.mt_cost_fn(cb)
    rc = B.load().mt_playoff_pointers(n, arr(lens), n_stages, arr(flat), costs, len(recs), top_k, fn, None, best, C.byref(bc), C.byref(nev))
    assert rc == 0, B.load().mt_last_error()
    assert nev.value == len(seen)
    return [[best[i * P + j] for j in range(P)] for i in range(n)], bc.value, seen


def test_record_memory_round_trips_through_a_file_and_feeds_the_playoff(tmp_path):
    from paper_2111_14255_amd import api
    lens = [9, 12]
    target = [[2, 6], [4, 8]]
    rho, c, recs = lib_search(lens, 3, 3, 4, 5, B.MT_SEARCH_COORDINATE, _cost(target))
    path = str(tmp_path / "records.json")
    api.save_records(path, lens, 3, recs, note="unit test")
    lens2, n_stages2, recs2 = api.load_records(path)
    assert (lens2, n_stages2, recs2) == (lens, 3, recs)
    # the stored memory is all the play-off needs: same winner as on the live records, and as the oracle's rule
    final = lambda r: _cost(target)(r) + 0.25
    got = lib_playoff(lens2, n_stages2, recs2, 3, final)
    assert got[:2] == lib_playoff(lens, 3, recs, 3, final)[:2] == S.playoff(lens, 2, recs, 3, final)[:2]
    # a file whose matrices do not fit the operator counts is refused
    import json
    doc = json.load(open(path))
    doc["records"][0]["pointers"][0] = [7, 3]
    json.dump(doc, open(path, "w"))
    with pytest.raises(ValueError):
        api.load_records(path)


def test_playoff_matches_oracle_and_can_overturn_the_first_measurement():
    lens = [23, 21, 54]
    target = [[5, 11, 17], [3, 9, 20], [10, 30, 50]]
    _, _, recs = S.coordinate_descent(lens, 3, 2, 4, _cost(target), 11, seed_baselines=True)
    recs = recs + [recs[3]]                                       # a duplicate matrix must be measured once only
    one_stage = [[n] * 3 for n in lens]
    # second measurement: the noisy first one is replaced by a cost that prefers the one-stage matrix, then the third-best record
    order = sorted(range(len(recs)), key=lambda j: (recs[j][1], j))
    third = recs[order[2]][0]
    final = lambda rho: 1.0 if rho == one_stage else 2.0 if rho == third else 3.0 + _cost(target)(rho)
    for top_k in (1, 3, 5):
        rho, c, seen = lib_playoff(lens, 4, recs, top_k, final)
        orho, oc, oscored = S.playoff(lens, 3, recs, top_k, final)
        assert rho == orho and c == oc and seen == [m for m, _ in oscored]
        assert rho == one_stage and c == 1.0 and seen[-1] == one_stage and len(seen) == top_k + 1
    # without the one-stage preference the winner is the best of the second measurements, not of the first
    final2 = lambda rho: 2.0 if rho == third else 3.0 + _cost(target)(rho)
    rho, c, seen = lib_playoff(lens, 4, recs, 3, final2)
    assert (rho, c) == S.playoff(lens, 3, recs, 3, final2)[:2] and rho == third
    # the one-stage matrix is not measured twice when it is already among the leaders; ties go to the earlier candidate
    recs2 = [(one_stage, 0.1)] + recs
    rho, c, seen = lib_playoff(lens, 4, recs2, 2, lambda r: 5.0)
    assert seen.count(one_stage) == 1 and rho == one_stage and len(seen) == 2
    assert (rho, c) == S.playoff(lens, 3, recs2, 2, lambda r: 5.0)[:2]


def test_single_stage_search_is_trivial():
    rho, c, recs = lib_search([4, 5], 1, 1, 2, 5, B.MT_SEARCH_COORDINATE, lambda r: 3.0)
    assert rho == [[], []] and c == 3.0


def test_fold_bn_matches_oracle_bitwise():
    m = zoo.resnet18("f16", 1)
    raw = weights.make_params(m, 5, 0)
    for p in raw[:6]:
        if p is None or p["bn"] is None:
            continue
        w1, b1 = api.fold_bn(p["w"], p["bn"])
        w2, b2 = ofold.fold_bn(p["w"], p["bn"])
        np.testing.assert_array_equal(w1, w2)
        np.testing.assert_array_equal(b1, b2)


def test_storage_casts_match_oracle_rounding():
    v = (np.random.default_rng(3).standard_normal(5000) * np.exp(np.random.default_rng(4).uniform(-20, 12, 5000))).astype(np.float32)
    for dt in ("f16", "bf16"):
        with np.errstate(over="ignore"):
            mine = api.from_storage(api.to_storage(v, dt), dt)
        np.testing.assert_array_equal(mine, oops.round_array(v, dt))


@pytest.mark.parametrize("name", ["tinyA", "tinyB", "tinyC", "tinyD", "resnet18", "resnet50", "vgg16", "mobilenetv2", "alexnet",
                                  "alexnet_published", "inceptionv3"])
def test_shape_inference_matches_model_tables(name):
    spec = zoo.BUILDERS[name]("f16", 2)
    m = api.Model(spec)
    assert m.num_ops() == len(spec.ops)
    flops = 0
    for i, op in enumerate(spec.ops):
        info = m.op_info(i)
        assert (info.in_h, info.in_w, info.in_c) == tuple(op.in_shape)
        assert (info.out_h, info.out_w, info.out_c) == tuple(op.out_shape)
        if op.kind in ("conv", "dwconv", "fc"):        # the MAC-counting kinds; normalisation and add report their own count
            flops += info.flops
        assert info.bytes > 0
    assert flops == 2 * spec.macs()
    assert m.out_features() == spec.out_features
    assert m.arena_bytes() > 0


def _model(ops, dtype=B.MT_F16, dims=(1, 8, 8, 8)):
    lib = B.load()
    h = C.c_void_p()
    assert lib.mt_model_begin(dtype, *dims, C.byref(h)) == 0
    for d in ops:
        assert lib.mt_model_add_op(h, C.byref(d), None) == 0
    rc = lib.mt_model_end(h)
    lib.mt_model_destroy(h)
    return rc


def _op(kind=B.MT_CONV, src=0, res=-1, dst=1, oc=8, coff=0, ctot=0, r=3, s=3, sh=1, sw=1, ph=1, pw=1, act=0, groups=1):
    return B.mt_op_desc(kind, src, res, dst, oc, coff, ctot, r, s, sh, sw, ph, pw, act, groups, 1e-4, 0.75, 2.0)


def test_model_validation_errors():
    lib = B.load()
    assert _model([_op()]) == 0
    assert _model([_op(src=3)]) == B.MT_ERR_SHAPE_MISMATCH            # input never produced
    assert _model([_op(r=11, s=11, ph=0, pw=0)]) == B.MT_ERR_SHAPE_MISMATCH   # window larger than input
    assert _model([_op(ph=3)]) == B.MT_ERR_SHAPE_MISMATCH              # pad >= window
    assert _model([_op(res=2)]) == B.MT_ERR_SHAPE_MISMATCH             # residual never produced
    assert _model([_op(), _op(src=1, dst=2, oc=4, res=1)]) == 0        # residual wider than the output is allowed
    assert _model([_op(), _op(src=1, dst=2, oc=16, res=1)]) == B.MT_ERR_SHAPE_MISMATCH
    assert _model([_op(coff=4, ctot=8)]) == B.MT_ERR_SHAPE_MISMATCH    # channel range exceeds the tensor
    assert _model([_op(dst=1, ctot=16), _op(dst=1, coff=8, ctot=16, sh=2, sw=2)]) == B.MT_ERR_SHAPE_MISMATCH
    assert _model([_op(kind=B.MT_MAXPOOL, res=0)]) == B.MT_ERR_SHAPE_MISMATCH
    assert _model([]) == B.MT_ERR_SHAPE_MISMATCH
    assert _model([_op(dst=1 << 30)]) == B.MT_ERR_SHAPE_MISMATCH       # tensor id far beyond what one operator can define
    assert _model([_op(groups=3)]) == B.MT_ERR_SHAPE_MISMATCH                      # 8 channels do not split into 3 groups
    assert _model([_op(groups=2)]) == 0
    assert _model([_op(kind=B.MT_MAXPOOL, groups=2)]) == B.MT_ERR_SHAPE_MISMATCH   # groups on a pool
    assert _model([_op(kind=B.MT_LRN, r=4)]) == B.MT_ERR_SHAPE_MISMATCH            # even window
    assert _model([_op(kind=B.MT_LRN, r=5)]) == 0
    assert _model([_op(kind=B.MT_ADD)]) == B.MT_ERR_SHAPE_MISMATCH                 # no second summand
    assert _model([_op(oc=8), _op(kind=B.MT_ADD, src=1, res=0, dst=2)]) == 0
    assert _model([_op(oc=16), _op(kind=B.MT_ADD, src=1, res=0, dst=2)]) == B.MT_ERR_SHAPE_MISMATCH   # 16 + 8 channels
    # 32-bit offsets inside the kernels: a tensor of 2 GiB or more is refused when the model is finalised
    assert _model([_op(oc=64)], dims=(64, 512, 512, 64)) == B.MT_ERR_SHAPE_MISMATCH        # 2 GiB fp16 input and output
    assert "2 GiB" in lib.mt_last_error().decode()
    assert _model([_op(oc=64)], dims=(32, 512, 512, 63)) == 0                              # just below
    h = C.c_void_p()
    assert lib.mt_model_begin(7, 1, 8, 8, 8, C.byref(h)) == B.MT_ERR_INVALID_ARG
    assert lib.mt_model_begin(B.MT_F16, 0, 8, 8, 8, C.byref(h)) == B.MT_ERR_INVALID_ARG
    assert lib.mt_model_end(None) == B.MT_ERR_INVALID_ARG


def test_set_weights_checks_sizes():
    lib = B.load()
    h = C.c_void_p()
    assert lib.mt_model_begin(B.MT_F16, 1, 8, 8, 8, C.byref(h)) == 0
    d = _op()
    assert lib.mt_model_add_op(h, C.byref(d), None) == 0
    w = np.zeros(8 * 3 * 3 * 8, dtype=np.float16)
    assert lib.mt_model_set_weights(h, 0, w.ctypes.data_as(C.c_void_p), w.nbytes, None, 0) == B.MT_ERR_NOT_FINALIZED
    assert lib.mt_model_end(h) == 0
    assert lib.mt_model_set_weights(h, 0, w.ctypes.data_as(C.c_void_p), w.nbytes - 2, None, 0) == B.MT_ERR_SHAPE_MISMATCH
    b = np.zeros(7, dtype=np.float32)
    assert lib.mt_model_set_weights(h, 0, w.ctypes.data_as(C.c_void_p), w.nbytes, b.ctypes.data_as(C.POINTER(C.c_float)), 7) == B.MT_ERR_SHAPE_MISMATCH
    assert lib.mt_model_set_weights(h, 0, w.ctypes.data_as(C.c_void_p), w.nbytes, None, 0) == 0
    assert lib.mt_model_set_weights(h, 1, w.ctypes.data_as(C.c_void_p), w.nbytes, None, 0) == B.MT_ERR_INVALID_ARG
    lib.mt_model_destroy(h)


def test_speedup_definition_matches_printed_tables():
    from bench import speedup
    with open(os.path.join(ROOT, "tests", "golden", "speedups.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 12
    for seq, ours, printed in rows:
        assert abs(speedup(float(seq), float(ours)) - float(printed)) < 0.01   # printed to two decimals, some rounded, some truncated


def test_cu_share_descent_matches_oracle():
    target = [64, 160, 32]
    calls = []

    def cost(sh):
        return float(sum(abs((a or 256) - b) for a, b in zip(sh, target))) + 1.0

    def cb(ptr, _u):
        v = [ptr[i] for i in range(3)]
        calls.append(v)
        return cost(v)

    best = (I32 * 3)()
    bc = C.c_double(cost([0, 0, 0]))
    fn = B.mt_share_cost_fn(cb)
    assert B.load().mt_search_cu_share(3, 256, 2, fn, None, best, C.byref(bc)) == 0
    ocalls = []
    oshare, ocost = S.cu_share_descent(3, 256, 2, lambda sh: (ocalls.append(list(sh)) or cost(sh)), cost([0, 0, 0]))
    assert [best[i] for i in range(3)] == oshare == [64, 160, 32]
    assert bc.value == ocost and calls == ocalls


def test_cu_share_descent_from_a_start_vector():
    target = [32, 160, 64]

    def cost(sh):
        return float(sum(abs((a or 256) - b) for a, b in zip(sh, target))) + 1.0

    start = [64, 96, 96]
    best = (I32 * 3)(*start)
    bc = C.c_double(cost(start))
    calls, ocalls = [], []
    fn = B.mt_share_cost_fn(lambda ptr, _u: (calls.append([ptr[i] for i in range(3)]) or cost(calls[-1])))
    assert B.load().mt_search_cu_share(3, 256, 1, fn, None, best, C.byref(bc)) == 0
    oshare, ocost = S.cu_share_descent(3, 256, 1, lambda sh: (ocalls.append(list(sh)) or cost(sh)), cost(start), start)
    assert [best[i] for i in range(3)] == oshare == target
    assert bc.value == ocost == 1.0 and calls == ocalls
    bad = (I32 * 3)(64, 300, 0)
    assert B.load().mt_search_cu_share(3, 256, 1, fn, None, bad, C.byref(bc)) != 0


def test_proportional_cu_share():
    lib = B.load()

    def host(w, cus=256):
        out = (I32 * len(w))()
        assert lib.mt_proportional_cu_share(len(w), cus, (C.c_double * len(w))(*w), out) == 0
        return [out[i] for i in range(len(w))]

    # hand-worked: 5 spare eighths, quotas 1.163 / 1.954 / 1.883 -> floors 1,1,1, the two left go to tenants 1 and 2
    assert host([147.0, 247.0, 238.0]) == [64, 96, 96] == S.proportional_shares([147.0, 247.0, 238.0], 256)
    assert host([1.0, 1.0]) == [128, 128]
    assert host([3.0, 1.0]) == [192, 64]     # 6 spare eighths, quotas 4.5 / 1.5: tie on the remainder, lower index first
    assert host([0.0, 0.0, 0.0]) == [96, 96, 64] == S.proportional_shares([0.0, 0.0, 0.0], 256)
    assert host([1.0] * 8) == [32] * 8
    assert host([5.0] * 12) == [32] * 12 == S.proportional_shares([5.0] * 12, 256)
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(1, 9))
        w = [float(x) for x in rng.uniform(0.0, 10.0, n)]
        sh = host(w)
        assert sh == S.proportional_shares(w, 256)
        assert sum(sh) == 256 and min(sh) >= 32 and all(v % 32 == 0 for v in sh)
        for i in range(n):                                       # monotone: a heavier tenant never gets less
            for j in range(n):
                if w[i] > w[j]:
                    assert sh[i] >= sh[j]
    assert lib.mt_proportional_cu_share(3, 256, (C.c_double * 3)(1.0, -1.0, 1.0), (I32 * 3)()) != 0


def test_wave_priority_descent_matches_oracle_and_finds_a_separable_optimum():
    # a separable cost with a known minimum: the descent must land on it in one round and stop after the next one
    target = [3, 0, -1, 2]

    def cost(pr):
        return float(sum((a - b) ** 2 for a, b in zip(pr, target))) + 0.5

    for start in ([0, 0, 0, 0], [-1, 3, 2, 1]):
        best = (I32 * 4)(*start)
        bc = C.c_double(cost(start))
        calls, ocalls = [], []
        fn = B.mt_share_cost_fn(lambda ptr, _u: (calls.append([ptr[i] for i in range(4)]) or cost(calls[-1])))
        assert B.load().mt_search_wave_priority(4, 5, fn, None, best, C.byref(bc)) == 0
        oprio, ocost = S.wave_priority_descent(4, 5, lambda pr: (ocalls.append(list(pr)) or cost(pr)), cost(start), start)
        assert [best[i] for i in range(4)] == oprio == target
        assert bc.value == ocost == 0.5 and calls == ocalls
        assert len(calls) <= 2 * 4 * 5                      # one improving round, one round without change, then stop
    # a cost that never improves keeps the start vector and evaluates one round only
    best = (I32 * 2)(1, 2)
    bc = C.c_double(1.0)
    n = []
    fn = B.mt_share_cost_fn(lambda ptr, _u: (n.append(1) or 2.0))
    assert B.load().mt_search_wave_priority(2, 3, fn, None, best, C.byref(bc)) == 0
    assert [best[0], best[1]] == [1, 2] and bc.value == 1.0 and len(n) == 8
    bad = (I32 * 2)(0, 4)
    assert B.load().mt_search_wave_priority(2, 1, fn, None, bad, C.byref(bc)) != 0
