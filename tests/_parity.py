"""Lock-step comparison of the HIP library with the fp64 oracle on the same seeded chunks.

Output bar: max-abs error 2e-2 for bf16 streams, 1e-4 for fp32 streams.
Retained sets: identical, except that keys whose fp64 biased score lies within 1e-5
(relative) of the r-th largest may be swapped; after such a swap the oracle adopts the GPU's
set so that later steps stay comparable.
"""
import numpy as np
import torch

OUT_TOL = {torch.bfloat16: 2e-2, torch.float32: 1e-4}
BAND = 1e-5


def check_retained(I_gpu, I_orc, Wb, n, budget, recent, band=BAND):
    """I_gpu, I_orc: [Hkv, count] int arrays.  Wb: oracle biased scores [Hkv, c] or None.
    Returns the number of (in-band) swapped keys."""
    assert I_gpu.shape == I_orc.shape, (I_gpu.shape, I_orc.shape)
    count = I_gpu.shape[1]
    assert count == min(n, budget)
    assert (np.diff(I_gpu, axis=1) > 0).all(), "retained indices are not strictly ascending"
    assert I_gpu.min() >= 0 and I_gpu.max() < n
    keep_recent = min(recent, n)
    if keep_recent:
        assert (I_gpu[:, count - keep_recent:] == np.arange(n - keep_recent, n)).all(), "recent window not retained"
    swaps = 0
    for h in range(I_gpu.shape[0]):
        g, o = set(I_gpu[h].tolist()), set(I_orc[h].tolist())
        if g == o:
            continue
        assert Wb is not None, "sets differ in a step that does not evict"
        r = budget - recent
        wr = np.sort(Wb[h])[::-1][r - 1]                      # r-th largest fp64 score
        diff = np.array(sorted(g ^ o))
        off = np.abs(Wb[h][diff] - wr)
        assert (off <= band * abs(wr)).all(), (
            "head %d: retained sets differ outside the tie band: idx %s, |W-W_r| %s, W_r %g"
            % (h, diff[:8], off[:8], wr))
        swaps += len(diff) // 2
    return swaps


class LockStep:
    """Drives a binding.Stream and an OracleStream with the same chunks."""

    def __init__(self, gpu, oracle, band=BAND):
        self.gpu, self.oracle, self.band = gpu, oracle, band
        self.swaps = 0
        self.max_err = 0.0
        self.steps = 0

    def step(self, q, k, v, check_state=False, strict=False):
        """strict: the retained sets must be identical, ties included (for inputs whose ties are exact on
        both sides, where the band of check_retained would hide a wrong choice among them)."""
        dev = self.gpu.device
        out_g, ret_g, n_g = self.gpu.step(q.to(dev), k.to(dev), v.to(dev))
        t = len(self.oracle)
        out_o = self.oracle.attend(q.double().numpy(), k.double().numpy(), v.double().numpy())
        n = t + q.shape[0]
        err = float(np.abs(out_g.double().cpu().numpy() - out_o).max())
        self.max_err = max(self.max_err, err)
        assert np.isfinite(err) and err <= OUT_TOL[self.gpu.dtype], "step %d: attention output off by %g" % (self.steps, err)
        count = int(n_g.item())
        assert count == min(n, self.gpu.budget) == len(self.gpu)
        sc = self.oracle.scores()
        I_o = self.oracle.select()
        I_g = ret_g.cpu().numpy()[:, :count]
        self.swaps += check_retained(I_g, I_o, None if sc is None else sc[1], n, self.gpu.budget, self.gpu.recent,
                                     self.band)
        if strict:
            assert (I_g == I_o).all(), "step %d: retained lists differ at %s" % (self.steps, np.argwhere(I_g != I_o)[:4])
        self.oracle.commit(I_g)
        if check_state:
            self.check_state()
        self.steps += 1
        return out_g, I_g

    def attend(self, q, k, v):
        """First half of a layer-batched step: step_attend on the GPU, attend on the oracle, outputs
        compared.  If nothing is pending afterwards the step is finished here; otherwise finish()
        must follow the batched eviction."""
        dev = self.gpu.device
        self._t = len(self.oracle)
        out_g, self._ret, self._cnt = self.gpu.step_attend(q.to(dev), k.to(dev), v.to(dev))
        out_o = self.oracle.attend(q.double().numpy(), k.double().numpy(), v.double().numpy())
        self._n = self._t + q.shape[0]
        err = float(np.abs(out_g.double().cpu().numpy() - out_o).max())
        self.max_err = max(self.max_err, err)
        assert np.isfinite(err) and err <= OUT_TOL[self.gpu.dtype], "step %d: attention output off by %g" % (self.steps, err)
        assert self.gpu.pending == (self._n > self.gpu.budget)
        if not self.gpu.pending:
            self.finish()
        return out_g

    def finish(self):
        """Second half: the retained lists (written by step_attend or by the batched eviction)."""
        n = self._n
        count = int(self._cnt.item())
        assert count == min(n, self.gpu.budget) == len(self.gpu)
        sc = self.oracle.scores()
        I_o = self.oracle.select()
        I_g = self._ret.cpu().numpy()[:, :count]
        self.swaps += check_retained(I_g, I_o, None if sc is None else sc[1], n, self.gpu.budget, self.gpu.recent,
                                     self.band)
        self.oracle.commit(I_g)
        self.steps += 1
        return I_g

    def decode(self, q, k, v):
        """One decoding step on both sides (q [1,Hq,d], k/v [1,Hkv,d]); compares the outputs."""
        dev = self.gpu.device
        out_g = self.gpu.decode(q.to(dev), k.to(dev), v.to(dev))
        out_o = self.oracle.decode(q.double().numpy(), k.double().numpy(), v.double().numpy())
        err = float(np.abs(out_g.double().cpu().numpy() - out_o).max())
        self.max_err = max(self.max_err, err)
        assert np.isfinite(err) and err <= OUT_TOL[self.gpu.dtype], "decode step: attention output off by %g" % err
        assert len(self.gpu) == len(self.oracle) and self.gpu.streamed == self.oracle.streamed
        return out_g

    def adopt_gpu_state(self):
        """Spot-check protocol for late steps: the oracle takes over the GPU's exported cache."""
        K, V, pos, _ = self.gpu.export()
        self.oracle.load(K.double().cpu().numpy(), V.double().cpu().numpy(), pos.cpu().numpy(), self.gpu.streamed)

    def gpu_only(self, q, k, v):
        dev = self.gpu.device
        return self.gpu.step(q.to(dev), k.to(dev), v.to(dev))

    def check_state(self):
        K, V, pos, score = self.gpu.export()
        Ko, Vo, po = self.oracle.export()
        assert (pos.cpu().numpy() == po).all(), "stream positions differ"
        assert (K.double().cpu().numpy() == Ko).all() and (V.double().cpu().numpy() == Vo).all(), "cache rows differ"
        assert (self.gpu.positions().cpu().numpy() == po).all()
