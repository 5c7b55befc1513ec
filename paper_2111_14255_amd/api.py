"""Convenience layer over the C ABI: marshals model descriptions, weights and torch device buffers.

Every computation on the forward path happens inside libmtsched.so; this module only converts arguments.
PyTorch owns the device memory (arenas, inputs, outputs) and hands raw pointers to the library.
"""
import ctypes as C
import os

import numpy as np

from . import binding as B

_DT = {"f32": B.MT_F32, "f16": B.MT_F16, "bf16": B.MT_BF16}
_KIND = {"conv": B.MT_CONV, "dwconv": B.MT_DWCONV, "maxpool": B.MT_MAXPOOL, "avgpool": B.MT_AVGPOOL,
         "gap": B.MT_GLOBAL_AVGPOOL, "fc": B.MT_FC, "lrn": B.MT_LRN, "add": B.MT_ADD}
_ACT = {"none": B.MT_ACT_NONE, "relu": B.MT_ACT_RELU, "relu6": B.MT_ACT_RELU6}


def to_storage(a, dtype):
    """float32 array -> array holding the storage type's bits; the rounding itself is the library's (mt_round_to_storage)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    out = np.empty(a.shape, dtype=np.float16 if dtype == "f16" else np.uint16)
    B.check(B.load().mt_round_to_storage(a.ctypes.data_as(C.POINTER(C.c_float)), a.size, _DT[dtype], C.c_void_p(out.ctypes.data)))
    return out


def from_storage(a, dtype):
    """Inverse view: storage bits -> float32 values."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32)
    if dtype == "f16":
        return np.asarray(a).view(np.float16).astype(np.float32)
    return (np.asarray(a).view(np.uint16).astype(np.uint32) << 16).view(np.float32)


def save_records(path, lens, n_stages, records, note=""):
    """Writes the record memory D of a search (Alg. 1: every profiled pointer matrix with its cost) as JSON, so that
    the search can be audited or its leaders measured again later (Context.replay_records)."""
    import json
    doc = {"lens": [int(v) for v in lens], "n_stages": int(n_stages), "note": note,
           "records": [{"pointers": [[int(v) for v in row] for row in rho], "cost_ms": float(c)} for rho, c in records]}
    with open(path, "w") as f:
        json.dump(doc, f)


def load_records(path):
    """Returns (lens, n_stages, records) as written by save_records; checks that every matrix fits the operator counts."""
    import json
    with open(path) as f:
        doc = json.load(f)
    lens, n_stages = [int(v) for v in doc["lens"]], int(doc["n_stages"])
    records = []
    for r in doc["records"]:
        rho = [[int(v) for v in row] for row in r["pointers"]]
        if len(rho) != len(lens) or any(len(row) != n_stages - 1 for row in rho):
            raise ValueError("record does not match lens / n_stages")
        for row, n in zip(rho, lens):
            if any(v < 0 or v > n for v in row) or any(b < a for a, b in zip(row, row[1:])):
                raise ValueError("record holds an infeasible pointer row")
        records.append((rho, float(r["cost_ms"])))
    return lens, n_stages, records


def torch_dtype(dtype):
    import torch
    return {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[dtype]


def fold_bn(w, bn):
    """BN folding through the library's helper (fp32, before the cast to the storage type)."""
    w = np.ascontiguousarray(w, dtype=np.float32).copy()
    k = w.shape[0]
    bias = np.zeros(k, dtype=np.float32)
    fp = C.POINTER(C.c_float)
    arrs = [np.ascontiguousarray(bn[n], dtype=np.float32) for n in ("gamma", "beta", "mean", "var")]
    B.check(B.load().mt_fold_bn(w.ctypes.data_as(fp), k, w.size // k, *[x.ctypes.data_as(fp) for x in arrs],
                                C.c_float(bn["eps"]), bias.ctypes.data_as(fp)))
    return w, bias


class Model:
    """Host-side model handle built from a serial operator list (any object with the OpSpec fields)."""

    def __init__(self, spec, raw_params=None):
        lib = B.load()
        self.spec = spec
        self.dtype = spec.dtype
        self.h = C.c_void_p()
        B.check(lib.mt_model_begin(_DT[spec.dtype], spec.batch, spec.in_h, spec.in_w, spec.in_c, C.byref(self.h)))
        for op in spec.ops:
            d = B.mt_op_desc(_KIND[op.kind], op.in_tensor, op.res_tensor, op.out_tensor, op.out_c, op.out_c_offset,
                             op.out_c_total, op.r, op.s, op.stride_h, op.stride_w, op.pad_h, op.pad_w, _ACT[op.act],
                             getattr(op, "groups", 1), getattr(op, "lrn_alpha", 0.0), getattr(op, "lrn_beta", 0.0),
                             getattr(op, "lrn_k", 0.0))
            B.check(lib.mt_model_add_op(self.h, C.byref(d), None))
        B.check(lib.mt_model_end(self.h))
        if raw_params is not None:
            self.set_params(raw_params)

    def set_params(self, raw_params):
        lib = B.load()
        for i, p in enumerate(raw_params):
            if p is None:
                continue
            w, b = p["w"], p["bias"]
            if p.get("bn") is not None:
                w, b = fold_bn(w, p["bn"])
            ws = to_storage(w, self.dtype)
            bp = None if b is None else np.ascontiguousarray(b, dtype=np.float32)
            B.check(lib.mt_model_set_weights(self.h, i, ws.ctypes.data_as(C.c_void_p), ws.nbytes,
                                             None if bp is None else bp.ctypes.data_as(C.POINTER(C.c_float)),
                                             0 if bp is None else bp.size))

    def num_ops(self):
        n = C.c_int32()
        B.check(B.load().mt_model_num_ops(self.h, C.byref(n)))
        return n.value

    def op_info(self, i):
        info = B.mt_op_info()
        B.check(B.load().mt_model_op_info(self.h, i, C.byref(info)))
        return info

    def out_features(self):
        n = C.c_int64()
        B.check(B.load().mt_model_out_features(self.h, C.byref(n)))
        return n.value

    def arena_bytes(self):
        n = C.c_size_t()
        B.check(B.load().mt_model_arena_bytes(self.h, C.byref(n)))
        return n.value

    def close(self):
        if self.h:
            B.load().mt_model_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Schedule:
    def __init__(self, ctx, handle, pointers, n_stages, label=""):
        self.ctx, self.h, self.pointers, self.n_stages, self.label = ctx, handle, pointers, n_stages, label

    def set_wave_priority(self, prio):
        """prio: one entry per tenant, 0..3 or -1 (short kernels 3, others 0)."""
        arr = (C.c_int32 * len(prio))(*prio)
        B.check(B.load().mt_schedule_set_wave_priority(self.h, arr))

    def close(self):
        if self.h:
            B.load().mt_schedule_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Context:
    def __init__(self, device=0):
        import torch
        self.torch = torch
        self.lib = B.load()
        self.h = C.c_void_p()
        B.check(self.lib.mt_create(device, C.byref(self.h)))
        self.device = torch.device("cuda", device)
        self.arenas = []
        self.specs = []
        self.batch = []

    # -- tenants ---------------------------------------------------------------------------
    def register(self, model):
        nbytes = model.arena_bytes()
        arena = self.torch.empty(max(nbytes, 256) + 256, dtype=self.torch.uint8, device=self.device)
        base = (arena.data_ptr() + 255) // 256 * 256
        self.torch.cuda.synchronize(self.device)
        t = C.c_int32()
        B.check(self.lib.mt_register(self.h, model.h, C.c_void_p(base), nbytes, C.byref(t)))
        self.arenas.append(arena)
        self.specs.append(model.spec)
        return t.value

    def num_tenants(self):
        return len(self.specs)

    def lens(self):
        out = []
        for t in range(len(self.specs)):
            n = C.c_int32()
            B.check(self.lib.mt_tenant_num_ops(self.h, t, C.byref(n)))
            out.append(n.value)
        return out

    def op_info(self, tenant, i):
        info = B.mt_op_info()
        B.check(self.lib.mt_tenant_op_info(self.h, tenant, i, C.byref(info)))
        return info

    def release_idle_streams(self):
        B.check(self.lib.mt_release_idle_streams(self.h))

    def peak_mfma(self, dtype="f16", iters=100000):
        """TFLOP/s of a register-only loop of 32x32x16 matrix instructions on every unit (mt_probe_peak_mfma)."""
        v = C.c_float()
        B.check(self.lib.mt_probe_peak_mfma(self.h, _DT[dtype], iters, C.byref(v)))
        return v.value

    def peak_stream(self, mode="copy", nbytes=1 << 32, reps=10, groups_per_unit=2):
        """GB/s of a plain copy (read + written bytes) or read kernel over `nbytes` bytes (mt_probe_peak_stream)."""
        v = C.c_float()
        B.check(self.lib.mt_probe_peak_stream(self.h, {"copy": 0, "read": 1}[mode], nbytes, groups_per_unit, reps, C.byref(v)))
        return v.value

    def device_info(self):
        d = B.mt_device_info()
        B.check(self.lib.mt_get_device_info(self.h, C.byref(d)))
        return d

    def read_tensor(self, tenant, tensor_id, shape):
        spec = self.specs[tenant]
        npdt = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[spec.dtype]
        buf = np.empty(shape, dtype=npdt)
        B.check(self.lib.mt_tenant_read_tensor(self.h, tenant, tensor_id, buf.ctypes.data_as(C.c_void_p), buf.nbytes))
        return from_storage(buf, spec.dtype).reshape(shape)

    # -- buffers ---------------------------------------------------------------------------
    def make_input(self, tenant, x_f32):
        """float32 NHWC numpy array -> device tensor in the tenant's storage type."""
        spec = self.specs[tenant]
        bits = to_storage(x_f32, spec.dtype)
        t = self.torch.from_numpy(bits.view(np.int16) if spec.dtype == "bf16" else bits)
        if spec.dtype == "bf16":
            t = t.view(self.torch.bfloat16)
        return t.to(self.device).contiguous()

    def make_output(self, tenant):
        spec = self.specs[tenant]
        p, q, c = spec.ops[-1].out_shape
        ctot = spec.ops[-1].out_c_total or c
        return self.torch.zeros((spec.batch, p * q * ctot), dtype=torch_dtype(spec.dtype), device=self.device)

    def output_to_numpy(self, tenant, out):
        self.torch.cuda.synchronize(self.device)
        return out.detach().float().cpu().numpy()

    # -- schedules -------------------------------------------------------------------------
    def schedule(self, pointers, n_stages, concurrency=None, cu_share=None, order=B.MT_ISSUE_BFS, flags=0, label="",
                 wave_priority=None):
        n = self.num_tenants()
        P = n_stages - 1
        flat = [int(v) for row in pointers for v in row] if P > 0 else []
        assert len(flat) == n * P
        arr = (C.c_int32 * max(1, len(flat)))(*flat)
        conc = None if concurrency is None else (C.c_int32 * n_stages)(*concurrency)
        if cu_share is not None and len(cu_share) and isinstance(cu_share[0], (list, tuple)):    # one row of shares per stage
            assert len(cu_share) == n_stages and all(len(r) == n for r in cu_share)
            cu_share = [int(v) for r in cu_share for v in r]
            flags |= B.MT_SCHED_SHARE_PER_STAGE
        share = None if cu_share is None else (C.c_int32 * len(cu_share))(*cu_share)
        h = C.c_void_p()
        B.check(self.lib.mt_schedule_create(self.h, n, n_stages, arr, conc, share, order, flags, C.byref(h)))
        sched = Schedule(self, h, [list(r) for r in pointers], n_stages, label)
        if wave_priority is not None:
            sched.set_wave_priority(wave_priority)
        return sched

    def sequential(self, **kw):
        """One stage, concurrency 1: tenants one after another on one stream."""
        return self.schedule([[] for _ in self.specs], 1, concurrency=[1], label="sequential", **kw)

    def all_concurrent(self, **kw):
        """One stage, one stream per tenant, no barriers: the hardware scheduler decides."""
        return self.schedule([[] for _ in self.specs], 1, label="all-concurrent", **kw)

    def bind(self, inputs, outputs):
        """Marshals the buffer pointers once; pass the result to run() in place of (inputs, outputs) in a loop."""
        n = self.num_tenants()
        ins = (C.c_void_p * n)(*[t.data_ptr() for t in inputs])
        outs = (C.c_void_p * n)(*[t.data_ptr() for t in outputs])
        return (ins, outs, B.mt_timings(), n, (inputs, outputs))          # the tensors stay referenced

    def run(self, sched, inputs, outputs=None):
        """One pass.  inputs / outputs: lists of device tensors, or the result of bind() as the only buffer argument."""
        ins, outs, tm, n, _ = inputs if outputs is None else self.bind(inputs, outputs)
        B.check(self.lib.mt_run(self.h, sched.h, ins, outs, C.byref(tm)))
        return {"makespan_ms": tm.makespan_ms, "host_issue_ms": tm.host_issue_ms, "n_launches": tm.n_launches,
                "stage_ms": [tm.stage_ms[i] for i in range(tm.n_stages)],
                "first_op_done_ms": [tm.first_op_done_ms[i] for i in range(n)], "n_fused": tm.n_fused,
                "tenant_done_ms": [tm.tenant_done_ms[i] for i in range(n)]}

    def run_static_scratch(self, sched, inputs, outputs=None):
        """One pass through mt_run_static_scratch (no device allocation; split workspaces in the library's fixed array)."""
        ins, outs, tm, n, _ = inputs if outputs is None else self.bind(inputs, outputs)
        B.check(self.lib.mt_run_static_scratch(self.h, sched.h, ins, outs, C.byref(tm)))
        return {"makespan_ms": tm.makespan_ms, "host_issue_ms": tm.host_issue_ms, "n_launches": tm.n_launches,
                "stage_ms": [tm.stage_ms[i] for i in range(tm.n_stages)], "n_fused": tm.n_fused}

    def run_makespan(self, sched, bound):
        """One pass on bound buffers; returns (makespan_ms, host_issue_ms) only: the cheap form for timing loops."""
        tm = bound[2]
        B.check(self.lib.mt_run(self.h, sched.h, bound[0], bound[1], C.byref(tm)))
        return tm.makespan_ms, tm.host_issue_ms

    def profile_ops(self, tenant, inp, out, repeats=5):
        n = self.lens()[tenant]
        ms = (C.c_float * n)()
        B.check(self.lib.mt_profile_ops(self.h, tenant, C.c_void_p(inp.data_ptr()), C.c_void_p(out.data_ptr()), repeats, ms))
        return [ms[i] for i in range(n)]

    def search(self, inputs, outputs, n_stages, rounds=2, candidates=6, runs=5, warmup=1, seed=1,
               algo=B.MT_SEARCH_COORDINATE, order=B.MT_ISSUE_BFS, flags=0, seed_baselines=True, cu_share_rounds=0,
               wave_priority_rounds=0, search_concurrency=False, playoff_top=0, playoff_runs=21):
        """Returns (pointer matrix, best cost, records), then the CU shares if cu_share_rounds > 0, then the wave
        priorities if wave_priority_rounds > 0, then the per-stage concurrency if search_concurrency."""
        n = self.num_tenants()
        P = n_stages - 1
        opts = B.mt_search_opts(algo, n_stages, rounds, candidates, runs, warmup, order, flags, 1 if seed_baselines else 0, cu_share_rounds,
                                wave_priority_rounds, 1 if search_concurrency else 0, playoff_top, playoff_runs, seed)
        cap = rounds * n * candidates + 2
        best = (C.c_int32 * max(1, n * P))()
        best_cost = C.c_double()
        shares = (C.c_int32 * n)()
        prio = (C.c_int32 * n)()
        conc = (C.c_int32 * n_stages)()
        recp = (C.c_int32 * max(1, cap * n * P))()
        recc = (C.c_double * cap)()
        nrec = C.c_int32()
        ins = (C.c_void_p * n)(*[t.data_ptr() for t in inputs])
        outs = (C.c_void_p * n)(*[t.data_ptr() for t in outputs])
        B.check(self.lib.mt_search(self.h, C.byref(opts), ins, outs, best, conc, shares, prio, C.byref(best_cost), recp, recc, cap,
                                  C.byref(nrec)))
        rho = [[best[i * P + j] for j in range(P)] for i in range(n)]
        records = [([[recp[(k * n + i) * P + j] for j in range(P)] for i in range(n)], recc[k]) for k in range(min(nrec.value, cap))]
        out = (rho, best_cost.value, records)
        if cu_share_rounds > 0:
            out += ([shares[i] for i in range(n)],)
        if wave_priority_rounds > 0:
            out += ([prio[i] for i in range(n)],)
        if search_concurrency:
            out += ([conc[i] for i in range(n_stages)],)
        return out

    def replay_records(self, records, n_stages, inputs, outputs, top_k=3, runs=21, warmup=2, flags=0, order=B.MT_ISSUE_BFS):
        """Play-off over a stored record memory (load_records): the top_k records of lowest stored cost and the
        one-stage matrix are profiled again on this context (median makespan of `runs` runs each); returns
        (pointer matrix, cost, number of matrices measured)."""
        n, P = self.num_tenants(), n_stages - 1
        lens = self.lens()
        bound = self.bind(inputs, outputs)

        def cost(ptr, _user):
            rho = [[ptr[i * P + j] for j in range(P)] for i in range(n)]
            s = self.schedule(rho, n_stages, order=order, flags=flags)
            try:
                for _ in range(warmup):
                    self.run(s, bound)
                v = sorted(self.run(s, bound)["makespan_ms"] for _ in range(runs))
            finally:
                s.close()
            return v[len(v) // 2]

        flat = [v for rho, _ in records for row in rho for v in row]
        costs = (C.c_double * max(1, len(records)))(*[c for _, c in records])
        best = (C.c_int32 * max(1, n * P))()
        bc, nev = C.c_double(), C.c_int32()
        fn = B.mt_cost_fn(cost)
        B.check(self.lib.mt_playoff_pointers(n, (C.c_int32 * n)(*lens), n_stages, (C.c_int32 * max(1, len(flat)))(*flat), costs,
                                             len(records), top_k, fn, None, best, C.byref(bc), C.byref(nev)))
        return [[best[i * P + j] for j in range(P)] for i in range(n)], bc.value, nev.value

    def close(self):
        if self.h:
            self.torch.cuda.synchronize(self.device)
            self.lib.mt_destroy(self.h)
            self.h = None
            self.arenas = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
