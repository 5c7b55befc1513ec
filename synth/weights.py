"""Seeded raw parameters and inputs.  Draws only: nothing here folds, rounds or computes.

Per operator the generator returns a dict of float32 arrays:
  conv   : w [K,R,S,C]  He-normal, std = sqrt(2 / (R*S*C))
  dwconv : w [C,R,S]    He-normal, std = sqrt(2 / (R*S))
  fc     : w [K,J]      He-normal, std = sqrt(2 / J)
  bias   : [K]  N(0, 0.05^2) for operators without BN, absent (None) with BN
  bn     : gamma ~ U[0.9,1.1]*gain, beta ~ N(0,0.1^2), mean ~ N(0,0.1^2), var ~ U[0.9,1.1]
Each (base seed, tenant, operator) owns an independent Philox stream, so two
tenants with the same architecture get different parameters.
"""
import numpy as np
from .graph import ModelSpec

BN_EPS = 1e-5


def _rng(seed, tenant, op_index, lane):
    key = np.array([np.uint64(seed), np.uint64((tenant << 40) | (op_index << 8) | lane)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def make_params(model: ModelSpec, seed: int, tenant: int):
    params = []
    for i, op in enumerate(model.ops):
        if op.kind not in ("conv", "dwconv", "fc"):
            params.append(None)
            continue
        h, w, c = op.in_shape
        g = _rng(seed, tenant, i, 0)
        if op.kind == "conv":
            cg = c // op.groups
            shape, fan_in = (op.out_c, op.r, op.s, cg), op.r * op.s * cg
        elif op.kind == "dwconv":
            shape, fan_in = (c, op.r, op.s), op.r * op.s
        else:
            shape, fan_in = (op.out_c, h * w * c), h * w * c
        wgt = (g.standard_normal(shape, dtype=np.float32) * np.float32(np.sqrt(2.0 / fan_in))).astype(np.float32)
        k = shape[0]
        p = {"w": wgt, "bias": None, "bn": None}
        g2 = _rng(seed, tenant, i, 1)
        if op.bn:
            p["bn"] = {
                "gamma": (g2.uniform(0.9, 1.1, k) * op.bn_gain).astype(np.float32),
                "beta": (g2.standard_normal(k) * 0.1).astype(np.float32),
                "mean": (g2.standard_normal(k) * 0.1).astype(np.float32),
                "var": g2.uniform(0.9, 1.1, k).astype(np.float32),
                "eps": BN_EPS,
            }
        else:
            p["bias"] = (g2.standard_normal(k) * 0.05).astype(np.float32)
        params.append(p)
    return params


def make_input(model: ModelSpec, seed: int, tenant: int, dist: str):
    g = _rng(seed, tenant, 0xFFFF, 2)
    shape = (model.batch, model.in_h, model.in_w, model.in_c)
    if dist == "uniform":
        return g.random(shape, dtype=np.float32)
    return g.standard_normal(shape, dtype=np.float32)
