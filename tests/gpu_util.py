"""Helpers for the GPU parity tests: upload seeded inputs, run the oracle, compare."""
import numpy as np
import torch

from paper_2506_03077_amd import binding as sb

TOL = {"f32": 1e-4, "bf16": 2e-2}      # norm-wise relative error bound per tensor


def tdtype(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def code(dtype):
    return sb.SBP_BF16 if dtype == "bf16" else sb.SBP_F32


def dev(a, dtype):
    """numpy (values already representable in dtype) -> device tensor of that dtype."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda").to(tdtype(dtype)).contiguous()


def host(t):
    return t.detach().to(torch.float64).cpu().numpy()


def relerr(got, want):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    den = np.linalg.norm(want)
    return float(np.linalg.norm(got - want) / den) if den > 0 else float(np.linalg.norm(got))


def assert_close(got, want, tol, name):
    e = relerr(got, want)
    assert np.isfinite(e) and e <= tol, f"{name}: norm-wise relative error {e:.3e} > {tol:.1e}"
    return e


def oracle_cfg(cfg):
    return dict(n_q_heads=cfg["n_q_heads"], n_kv_heads=cfg["n_kv_heads"], head_dim=cfg["head_dim"],
                rms_eps=cfg.get("rms_eps", 1e-6), rope_theta=cfg.get("rope_theta", 1e4),
                pos_offset=cfg.get("pos_offset", 0))


def lib_layer_cfg(cfg, seq_len, chunk, batch=1, grad_dtype="f32", dw_group_rows=0):
    return sb.layer_cfg(code(cfg["dtype"]), batch, seq_len, chunk, cfg["hidden"], cfg["n_q_heads"],
                        cfg["n_kv_heads"], cfg["head_dim"], cfg["mlp_width"], cfg.get("rms_eps", 1e-6),
                        cfg.get("rope_theta", 1e4), cfg.get("pos_offset", 0), code(grad_dtype), dw_group_rows)
