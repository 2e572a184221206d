"""Helpers for the GPU parity tests: upload seeded inputs, run the oracle, compare."""
import numpy as np
import torch

from paper_2506_03077_amd import binding as sb

TOL = {"f32": 1e-4, "bf16": 2e-2}      # relative error bound per tensor (norm-wise, and max-abs scaled by max|ref|)
BLOCK = 256                            # edge of the blocks of the per-block gate: the output tile of the MFMA GEMMs
BLOCK_SLACK = 4.0                      # a block's norm-wise error may be this many times the tensor's bound


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


def block_errors(got, want, block=BLOCK):
    """Norm-wise error of every block x block tile of the tensor seen as a matrix [prod(leading dims), last dim],
    each relative to the larger of the reference tile's norm and the norm a tile of the tensor's mean square would
    have (so that tiles of near-zero reference values are measured against the tensor's scale, not against nothing)."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    if want.ndim < 2:
        got, want = got.reshape(1, -1), want.reshape(1, -1)
    got, want = got.reshape(-1, got.shape[-1]), want.reshape(-1, want.shape[-1])
    R, Cn = want.shape
    pr, pc = (-R) % block, (-Cn) % block

    def tiles(a):
        a = np.pad(a, ((0, pr), (0, pc)))
        return (a.reshape((R + pr) // block, block, (Cn + pc) // block, block) ** 2).sum(axis=(1, 3))

    diff2, ref2 = tiles(got - want), tiles(want)
    floor2 = np.mean(want * want) * block * block
    den2 = np.maximum(ref2, floor2)
    # an all-zero reference: any deviation at all is an infinite error
    return np.sqrt(np.where(den2 > 0, diff2 / np.where(den2 > 0, den2, 1.0), np.where(diff2 > 0, np.inf, 0.0)))


def assert_close(got, want, tol, name):
    """Three gates: norm-wise error of the whole tensor <= tol; largest elementwise deviation <= tol * max|ref|; and the
    norm-wise error of every 256 x 256 tile <= BLOCK_SLACK * tol, so that one wrong output tile of a large tensor -
    which moves the whole-tensor norm by far less than tol - still fails."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, f"{name}: shape {got.shape} != {want.shape}"
    e = relerr(got, want)
    assert np.isfinite(e) and e <= tol, f"{name}: norm-wise relative error {e:.3e} > {tol:.1e}"
    ref_max = float(np.max(np.abs(want))) if want.size else 0.0
    if ref_max == 0.0:
        return e          # an all-zero reference has no scale: the norm of `got` itself was held to tol above
    dev_max = float(np.max(np.abs(got - want)))
    assert dev_max <= tol * ref_max, \
        f"{name}: max-abs error {dev_max:.3e} > {tol:.1e} * max|ref| = {tol * ref_max:.3e}"
    if True:
        be = block_errors(got, want)
        i = np.unravel_index(int(np.argmax(be)), be.shape)
        assert be[i] <= BLOCK_SLACK * tol, f"{name}: tile {i} of {be.shape} has norm-wise error {be[i]:.3e} > {BLOCK_SLACK * tol:.1e}"
    return e


def oracle_cfg(cfg):
    return dict(n_q_heads=cfg["n_q_heads"], n_kv_heads=cfg["n_kv_heads"], head_dim=cfg["head_dim"],
                rms_eps=cfg.get("rms_eps", 1e-6), rope_theta=cfg.get("rope_theta", 1e4),
                pos_offset=cfg.get("pos_offset", 0), window=cfg.get("window", 0))


def lib_layer_cfg(cfg, seq_len, chunk, batch=1, grad_dtype="f32", dw_group_rows=0, seq_first=None):
    return sb.layer_cfg(code(cfg["dtype"]), batch, seq_len, chunk, cfg["hidden"], cfg["n_q_heads"],
                        cfg["n_kv_heads"], cfg["head_dim"], cfg["mlp_width"], cfg.get("rms_eps", 1e-6),
                        cfg.get("rope_theta", 1e4), cfg.get("pos_offset", 0), code(grad_dtype), dw_group_rows,
                        cfg.get("window", 0), seq_first)
