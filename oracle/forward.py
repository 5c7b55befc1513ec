"""Forward pass of one tenant on the CPU oracle.  Test infrastructure only.

Walks the tenant's serial operator list (paper Sec. III-B, Eq. 1) and applies
the textbook definition of each operator.  The result is the same for every
schedule, because a schedule only changes when an operator runs (Sec. III-A:
operators of one model keep their data-flow order, models are independent).
"""
import numpy as np
from . import ops, fold


def prepare_params(model, raw_params):
    """Fold BN (float32), then round weights to the storage type.  Bias stays float32."""
    out = []
    for op, p in zip(model.ops, raw_params):
        if p is None:
            out.append(None)
            continue
        w, b = p["w"], p["bias"]
        if p["bn"] is not None:
            w, b = fold.fold_bn(w, p["bn"])
        out.append((ops.round_array(w, model.dtype), None if b is None else np.ascontiguousarray(b, np.float32)))
    return out


def forward(model, params, x, keep=False):
    """x: float32 [N,H,W,C] (rounded to the storage type here).  Returns the
    last operator's tensor as [N, features]; with keep=True also every tensor."""
    dt = model.dtype
    t = {0: ops.round_array(x, dt)}
    assert t[0].shape == (model.batch, model.in_h, model.in_w, model.in_c)
    for op, p in zip(model.ops, params):
        xin = t[op.in_tensor]
        y = t.get(op.out_tensor)
        st, pd, kk = (op.stride_h, op.stride_w), (op.pad_h, op.pad_w), (op.r, op.s)
        co, ct = op.out_c_offset, op.out_c_total
        if op.kind == "conv":
            res = t[op.res_tensor] if op.res_tensor >= 0 else None
            y = ops.conv(xin, p[0], p[1], st, pd, op.act, res, dt, y, co, ct, op.groups)
        elif op.kind == "dwconv":
            y = ops.dwconv(xin, p[0], p[1], st, pd, op.act, dt, y, co, ct)
        elif op.kind == "maxpool":
            y = ops.maxpool(xin, kk, st, pd, dt, y, co, ct)
        elif op.kind == "avgpool":
            y = ops.avgpool(xin, kk, st, pd, dt, y, co, ct)
        elif op.kind == "gap":
            y = ops.global_avgpool(xin, dt, y, co, ct)
        elif op.kind == "fc":
            y = ops.fc(xin, p[0], p[1], op.act, dt)
        elif op.kind == "lrn":
            y = ops.lrn(xin, op.r, op.lrn_alpha, op.lrn_beta, op.lrn_k, dt)
        elif op.kind == "add":
            y = ops.add(xin, t[op.res_tensor], op.act, dt)
        else:
            raise ValueError(op.kind)
        t[op.out_tensor] = y
    last = t[model.ops[-1].out_tensor]
    out = last.reshape(last.shape[0], -1)
    return (out, t) if keep else out
