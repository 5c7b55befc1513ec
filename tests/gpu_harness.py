"""Shared helpers of the GPU parity tests: run a tenant mix through the library, and through the oracle."""
import numpy as np

from synth import weights
from oracle import forward as OF

TOL = {"f32": 1e-4, "f16": 2e-2, "bf16": 2e-2}     # max|err| <= TOL * max|ref|


class Mix:
    """A set of tenants registered in one library context, with seeded inputs on the device."""

    def __init__(self, specs, seed, input_dist="normal"):
        from paper_2111_14255_amd import api
        self.api = api
        self.specs = specs
        self.seed = seed
        self.raw = [weights.make_params(m, seed, t) for t, m in enumerate(specs)]
        self.x = [weights.make_input(m, seed, t, input_dist) for t, m in enumerate(specs)]
        self.ctx = api.Context(0)
        for m, raw in zip(specs, self.raw):
            model = api.Model(m, raw)
            self.ctx.register(model)
            model.close()
        self.inputs = [self.ctx.make_input(t, x) for t, x in enumerate(self.x)]
        self._oracle = None

    def run(self, sched, poison=True):
        outs = [self.ctx.make_output(t) for t in range(len(self.specs))]
        if poison:
            for o in outs:
                o.fill_(float("nan"))
        tm = self.ctx.run(sched, self.inputs, outs)
        return [self.ctx.output_to_numpy(t, o) for t, o in enumerate(outs)], tm

    def oracle(self):
        if self._oracle is None:
            self._oracle = [OF.forward(m, OF.prepare_params(m, raw), x) for m, raw, x in zip(self.specs, self.raw, self.x)]
        return self._oracle

    def close(self):
        self.ctx.close()


def assert_close(got, ref, dtype, what=""):
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(ref).all(), what
    assert np.isfinite(got).all(), what + ": non-finite GPU output"
    scale = float(np.abs(ref).max())
    err = float(np.abs(got.astype(np.float64) - ref.astype(np.float64)).max())
    assert err <= TOL[dtype] * max(scale, 1e-30), "%s: max|err| %.4g > %.1e * max|ref| %.4g" % (what, err, TOL[dtype], scale)
    return err / max(scale, 1e-30)
