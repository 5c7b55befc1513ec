"""Plain-data description of one tenant: a serial list of operators.

The paper (Sec. III-B, Eq. 1) represents each model as one serial operator
sequence; multi-branch models are serialised.  `ModelSpec.ops` is that
sequence.  Tensors are named by small integers; tensor 0 is the model input.
An operator may write its channels at an offset inside a wider tensor, which
is how channel concatenation is expressed without a copy.
"""
from dataclasses import dataclass, field
from typing import List, Dict, Tuple

KINDS = ("conv", "dwconv", "maxpool", "avgpool", "gap", "fc", "lrn", "add")
ACTS = ("none", "relu", "relu6")
DTYPES = ("f32", "f16", "bf16")


@dataclass
class OpSpec:
    kind: str
    in_tensor: int
    out_tensor: int
    out_c: int = 0            # conv / fc: output channels; others: = input channels
    r: int = 1
    s: int = 1
    stride_h: int = 1
    stride_w: int = 1
    pad_h: int = 0
    pad_w: int = 0
    act: str = "none"
    res_tensor: int = -1      # tensor added before the activation, -1 = none
    out_c_offset: int = 0     # first channel written inside the output tensor
    out_c_total: int = 0      # channel count of the output tensor (0 = out_c)
    bn: bool = False          # synthetic batch-norm follows (to be folded)
    bn_gain: float = 1.0      # multiplier on the synthetic BN gamma
    groups: int = 1           # conv: independent channel groups
    lrn_alpha: float = 0.0    # lrn: b = a / (lrn_k + lrn_alpha * sum of squares over r neighbouring channels) ** lrn_beta
    lrn_beta: float = 0.0
    lrn_k: float = 0.0
    # filled by the builder, for generators and reports (not consumed by either implementation)
    in_shape: Tuple[int, int, int] = (0, 0, 0)    # H, W, C of the input tensor
    out_shape: Tuple[int, int, int] = (0, 0, 0)   # P, Q, channels written


@dataclass
class ModelSpec:
    name: str
    dtype: str
    batch: int
    in_h: int
    in_w: int
    in_c: int
    ops: List[OpSpec] = field(default_factory=list)

    @property
    def out_features(self) -> int:
        p, q, c = self.ops[-1].out_shape
        return p * q * c

    def macs(self) -> int:
        """Multiply-accumulates of one forward pass (conv, depthwise, fc), whole batch."""
        total = 0
        for op in self.ops:
            h, w, c = op.in_shape
            p, q, k = op.out_shape
            if op.kind == "conv":
                total += p * q * k * op.r * op.s * (c // op.groups)
            elif op.kind == "dwconv":
                total += p * q * k * op.r * op.s
            elif op.kind == "fc":
                total += k * h * w * c
        return total * self.batch


def _pair(v):
    return (v, v) if isinstance(v, int) else tuple(v)


class GraphBuilder:
    """Appends operators in serial order and tracks tensor shapes (H, W, C)."""

    def __init__(self, name, dtype, batch, in_h, in_w, in_c):
        assert dtype in DTYPES
        self.m = ModelSpec(name, dtype, batch, in_h, in_w, in_c)
        self.shapes: Dict[int, Tuple[int, int, int]] = {0: (in_h, in_w, in_c)}
        self.next_id = 1

    def new_tensor(self) -> int:
        t = self.next_id
        self.next_id += 1
        return t

    def _emit(self, op: OpSpec, p, q, c_written):
        tot = op.out_c_total or c_written
        op.in_shape = self.shapes[op.in_tensor]
        op.out_shape = (p, q, c_written)
        prev = self.shapes.get(op.out_tensor)
        if prev is not None:
            assert prev == (p, q, tot), (prev, (p, q, tot))
        self.shapes[op.out_tensor] = (p, q, tot)
        self.m.ops.append(op)
        return op.out_tensor

    def _window(self, kind, src, out_c, k, stride, pad, act, res, dst, c_off, c_tot, bn, gain):
        r, s = _pair(k)
        sh, sw = _pair(stride)
        ph, pw = _pair(pad)
        h, w, c = self.shapes[src]
        p = (h + 2 * ph - r) // sh + 1
        q = (w + 2 * pw - s) // sw + 1
        if dst is None:
            dst = self.new_tensor()
        oc = out_c if kind == "conv" else c
        op = OpSpec(kind, src, dst, oc, r, s, sh, sw, ph, pw, act, res, c_off, c_tot, bn, gain)
        return self._emit(op, p, q, oc)

    def conv(self, src, out_c, k, stride=1, pad=0, act="relu", bn=False, gain=1.0,
             res=-1, dst=None, c_off=0, c_tot=0, groups=1):
        t = self._window("conv", src, out_c, k, stride, pad, act, res, dst, c_off, c_tot, bn, gain)
        assert self.shapes[src][2] % groups == 0 and out_c % groups == 0
        self.m.ops[-1].groups = groups
        return t

    def lrn(self, src, size=5, alpha=1e-4, beta=0.75, k=2.0):
        h, w, c = self.shapes[src]
        op = OpSpec("lrn", src, self.new_tensor(), c, size, 1, lrn_alpha=alpha, lrn_beta=beta, lrn_k=k)
        return self._emit(op, h, w, c)

    def add(self, src, other, act="none"):
        assert self.shapes[src] == self.shapes[other]
        h, w, c = self.shapes[src]
        op = OpSpec("add", src, self.new_tensor(), c, act=act, res_tensor=other)
        return self._emit(op, h, w, c)

    def dwconv(self, src, k=3, stride=1, pad=1, act="relu", bn=False, gain=1.0):
        return self._window("dwconv", src, 0, k, stride, pad, act, -1, None, 0, 0, bn, gain)

    def maxpool(self, src, k, stride, pad=0, dst=None, c_off=0, c_tot=0):
        return self._window("maxpool", src, 0, k, stride, pad, "none", -1, dst, c_off, c_tot, False, 1.0)

    def avgpool(self, src, k, stride, pad=0):
        return self._window("avgpool", src, 0, k, stride, pad, "none", -1, None, 0, 0, False, 1.0)

    def gap(self, src):
        h, w, c = self.shapes[src]
        op = OpSpec("gap", src, self.new_tensor(), c, h, w)
        return self._emit(op, 1, 1, c)

    def fc(self, src, out_c, act="none"):
        h, w, c = self.shapes[src]
        op = OpSpec("fc", src, self.new_tensor(), out_c, h, w, act=act)
        return self._emit(op, 1, 1, out_c)

    def done(self) -> ModelSpec:
        return self.m
