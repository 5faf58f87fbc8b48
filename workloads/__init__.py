"""Seeded synthetic inputs shaped like the paper's dense experiments (Sec. 5.1).

This module only draws random input matrices and names problem sizes.  It
contains none of the method's arithmetic (no compression, no tensor
generation, no noise function) and belongs to neither the HIP library's package
nor the CPU oracle's: the tests and the benchmark of both take their inputs from here.

The paper's dense workload: I=J=K, Gaussian CP factor matrices A,B,C (I x R),
Gaussian compression matrices U_p (L x I), V_p (M x J), W_p (N x K), cubic
blocks of edge d.  The five benchmark configurations add sigma=0.01 noise and
fix R, P, L and d as listed in CONFIGS.
"""
from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 0x231113693000


@dataclass(frozen=True)
class Config:
    name: str
    I: int
    J: int
    K: int
    R: int
    P: int
    L: int
    M: int
    N: int
    dI: int
    dJ: int
    dK: int
    dtype: str           # "f32" or "bf16": type of the X tile and of U,V,W as the kernels consume them;
                         # "f32s": fp32 data, contractions on the fp16 matrix cores with two-piece operands
    materialised: bool   # X resident in HBM (True) or generated tile by tile inside the kernel (False)
    sigma: float = 0.01
    index: int = 0

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def elements(self) -> int:
        return self.I * self.J * self.K

    @property
    def flops(self) -> int:
        """Algorithmic flops of the three-mode chain, each mode once at full extent."""
        PL = self.P * self.L
        return 2 * PL * (self.I * self.J * self.K + self.M * self.J * self.K + self.M * self.N * self.K)


def _cube(name, index, n, R, P, L, d, dtype, materialised):
    return Config(name, n, n, n, R, P, L, L, L, d, d, d, dtype, materialised, 0.01, index)


CONFIGS = {
    "cfg1": _cube("cfg1", 0, 128, 8, 4, 16, 128, "f32", True),
    "cfg2": _cube("cfg2", 1, 512, 16, 16, 32, 128, "f32", True),
    "cfg3": _cube("cfg3", 2, 1024, 32, 32, 64, 256, "f32", True),
    "cfg4": _cube("cfg4", 3, 4096, 64, 64, 64, 256, "f32", False),
    "cfg5": _cube("cfg5", 4, 10000, 32, 48, 50, 250, "bf16", False),
    # scaled-down twins of the two generated configurations (same awkward sizes, oracle-sized)
    "cfg4_twin": _cube("cfg4_twin", 5, 512, 64, 64, 64, 256, "f32", False),
    "cfg5_twin": _cube("cfg5_twin", 6, 500, 32, 48, 50, 250, "bf16", False),
}


def with_sigma(cfg: Config, sigma: float) -> Config:
    return replace(cfg, sigma=sigma)


def _normal(seed, stream, shape, std):
    g = np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, stream]))
    return (g.standard_normal(shape, dtype=np.float64) * std).astype(np.float32)


def cp_factors(cfg: Config):
    """A (I x R), B (J x R), C (K x R): iid N(0,1), float32, column-major."""
    A = np.asfortranarray(_normal(cfg.seed, 1, (cfg.R, cfg.I), 1.0).T)
    B = np.asfortranarray(_normal(cfg.seed, 2, (cfg.R, cfg.J), 1.0).T)
    C = np.asfortranarray(_normal(cfg.seed, 3, (cfg.R, cfg.K), 1.0).T)
    return A, B, C


def compression_matrices(cfg: Config):
    """Stacked U (P*L x I), V (P*M x J), W (P*N x K): iid N(0, 1/L) etc., float32, row-major,
    replica p in rows p*L .. p*L+L-1."""
    U = _normal(cfg.seed, 4, (cfg.P * cfg.L, cfg.I), cfg.L ** -0.5)
    V = _normal(cfg.seed, 5, (cfg.P * cfg.M, cfg.J), cfg.M ** -0.5)
    W = _normal(cfg.seed, 6, (cfg.P * cfg.N, cfg.K), cfg.N ** -0.5)
    return U, V, W


def small(name="tiny", index=100, I=24, J=20, K=28, R=3, P=3, L=5, M=4, N=6, dI=12, dJ=10, dK=7,
          dtype="f32", materialised=True, sigma=0.01) -> Config:
    """An arbitrary small non-cubic configuration for tests."""
    return Config(name, I, J, K, R, P, L, M, N, dI, dJ, dK, dtype, materialised, sigma, index)


# ---- Two-stage compression (Sec. 4.4): sparse first-stage matrices, dense second-stage replicas ----

@dataclass(frozen=True)
class TwoStage:
    """First stage I x J x K -> (alpha L) x (beta M) x (gamma N) with sparse U, V, W shared by all
    replicas, second stage with dense U'_p (L x alpha L) etc.  The paper leaves the sparsity pattern
    open; the inputs drawn here are sparse sign matrices with `nnz_per_col` entries +-1/sqrt(nnz_per_col)
    in every column, at distinct rows drawn uniformly (a standard compressed-sensing ensemble)."""
    base: Config
    alpha: int = 2
    beta: int = 2
    gamma: int = 2
    nnz_per_col: int = 4

    @property
    def A1(self) -> int:
        return self.alpha * self.base.L

    @property
    def B1(self) -> int:
        return self.beta * self.base.M

    @property
    def C1(self) -> int:
        return self.gamma * self.base.N

    @property
    def second(self) -> Config:
        """The dense multi-replica problem on the first stage's output (one block)."""
        b = self.base
        return replace(b, name=b.name + "_stage2", I=self.A1, J=self.B1, K=self.C1,
                       dI=self.A1, dJ=self.B1, dK=self.C1, materialised=True)


def sparse_sign_csr(seed, stream, rows, cols, nnz_per_col):
    """CSR arrays (rowptr int64 [rows+1], colidx int32, val float32) of a rows x cols matrix whose every
    column holds nnz_per_col entries +-1/sqrt(nnz_per_col) at distinct rows; columns sorted inside a row."""
    s = min(nnz_per_col, rows)
    g = np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, stream]))
    r = np.argsort(g.random((cols, rows)), axis=1)[:, :s].astype(np.int64)      # s distinct rows per column
    sign = np.where(g.random((cols, s)) < 0.5, -1.0, 1.0)
    c = np.repeat(np.arange(cols, dtype=np.int64), s)
    r = r.reshape(-1)
    v = (sign.reshape(-1) / np.sqrt(s)).astype(np.float32)
    order = np.lexsort((c, r))
    r, c, v = r[order], c[order], v[order]
    rowptr = np.zeros(rows + 1, dtype=np.int64)
    np.add.at(rowptr, r + 1, 1)
    return np.cumsum(rowptr), c.astype(np.int32), v


def first_stage_matrices(ts: TwoStage):
    """Sparse U (alpha L x I), V (beta M x J), W (gamma N x K) as CSR triples."""
    b = ts.base
    return (sparse_sign_csr(b.seed, 7, ts.A1, b.I, ts.nnz_per_col),
            sparse_sign_csr(b.seed, 8, ts.B1, b.J, ts.nnz_per_col),
            sparse_sign_csr(b.seed, 9, ts.C1, b.K, ts.nnz_per_col))


def second_stage_matrices(ts: TwoStage):
    """Stacked dense U' (P*L x alpha L), V' (P*M x beta M), W' (P*N x gamma N), iid N(0, 1/L) etc."""
    b = ts.base
    return (_normal(b.seed, 10, (b.P * b.L, ts.A1), b.L ** -0.5),
            _normal(b.seed, 11, (b.P * b.M, ts.B1), b.M ** -0.5),
            _normal(b.seed, 12, (b.P * b.N, ts.C1), b.N ** -0.5))
