"""Helpers for the GPU parity tests: numpy <-> torch marshalling in the library's layouts."""
import numpy as np
import torch

from paper_2311_13693_amd import exat
import workloads as wl


def to_dev_x(X, bf16=False):
    """numpy (I,J,K) array -> flat CUDA tensor in column-major order."""
    t = torch.from_numpy(np.ascontiguousarray(X.reshape(-1, order="F"))).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def to_dev_mat(U):
    return torch.from_numpy(np.ascontiguousarray(U, dtype=np.float32)).cuda()


def to_dev_factor(A):
    """numpy column-major (I, R) -> CUDA tensor of shape (R, I), element (i, r) at r*I + i."""
    return torch.from_numpy(np.ascontiguousarray(A.T, dtype=np.float32)).cuda()


def y_to_numpy(Y, cfg):
    return Y.detach().cpu().numpy().astype(np.float64).reshape((cfg.L, cfg.M, cfg.N, cfg.P), order="F")


def desc_of(cfg):
    return exat.make_desc(cfg.I, cfg.J, cfg.K, cfg.L, cfg.M, cfg.N, cfg.P, cfg.dI, cfg.dJ, cfg.dK,
                          {"bf16": exat.EXAT_BF16, "f32s": exat.EXAT_F32_SPLIT}.get(cfg.dtype, exat.EXAT_F32))


def plan_with_factors(cfg, U, V, W):
    plan = exat.Plan(desc_of(cfg))
    plan.set_factors(to_dev_mat(U), to_dev_mat(V), to_dev_mat(W))
    return plan


def gen_of(cfg, A, B, C, sigma=None):
    return exat.make_gen(to_dev_factor(A), to_dev_factor(B), to_dev_factor(C), cfg.seed,
                         cfg.sigma if sigma is None else sigma)
