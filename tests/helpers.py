"""Shared helpers of the GPU parity tests: oracle-side preparation of a
BitLinear case and upload of its inputs."""
import numpy as np

import oracle
import synth


class Case:
    """Latent weights, activations and every oracle result for one BitLinear."""

    def __init__(self, seed, M, N, K, layer=0, matrix=0, relu2=False, full=True):
        self.M, self.N, self.K = M, N, K
        self.W = synth.latent_weights(seed, N, K, layer=layer, matrix=matrix)
        self.X = synth.activations_bf16(seed, M, K, layer=layer, matrix=matrix, relu2=relu2)
        self.beta, mean64 = oracle.absmean_beta(self.W, return_mean64=True)
        assert oracle.beta_guard_ok(mean64), "beta too close to an fp32 rounding midpoint: change the seed"
        self.Wt = oracle.ternarize(self.W, self.beta)
        self.q, self.scale, self.rowsum = oracle.quant_act(self.X)
        if full:
            self.acc = oracle.matmul_i32(self.q, self.Wt)
            self.y = oracle.rescale(self.acc, self.beta, self.scale)

    def packed(self, layout):
        if layout == 3:
            return oracle.pack_kmajor(self.Wt)
        return oracle.pack_trit5(self.Wt) if layout == 2 else oracle.pack_padded(self.Wt, layout)


def to_dev(a, dev="cuda:0"):
    import torch
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:  # bf16 bit patterns
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    return torch.from_numpy(a).to(dev)


def assert_y_close(y_gpu, y_ref, tol=1e-6):
    """Relative error <= tol where the reference is non-zero; exact +0 elsewhere."""
    yg = np.asarray(y_gpu, dtype=np.float64)
    yr = np.asarray(y_ref, dtype=np.float64)
    nz = yr != 0
    assert np.all(np.abs(yg[nz] - yr[nz]) <= tol * np.abs(yr[nz])), \
        "max rel err %g" % float(np.max(np.abs(yg[nz] - yr[nz]) / np.abs(yr[nz])))
    assert np.all(yg[~nz] == 0)
