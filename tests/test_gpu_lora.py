"""GPU parity of the adapter mode (App. D, experiment setup: rank-32 low-rank adapters, adapter gradients only) against
the fp64 oracle of the adapted layer: dx and every dA, dB; MFMA path, shape-agnostic paths, partial adapter sets,
batches, masks, and the 7B widths at the bench's chunk size."""
import numpy as np
import pytest
import torch

from oracle import lora as o_lora
from paper_2506_03077_amd import binding as sb
from paper_2506_03077_amd import synth

from gpu_util import TOL, assert_close, dev, host, lib_layer_cfg, oracle_cfg

pytestmark = pytest.mark.gpu

MID16 = dict(dtype="bf16", hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=128, mlp_width=512)
BIG16 = dict(dtype="bf16", hidden=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, mlp_width=4096)
ODD16 = dict(dtype="bf16", hidden=72, n_q_heads=6, n_kv_heads=2, head_dim=24, mlp_width=172)
TINY = synth.CONFIGS["tiny"]


def make_adapters(cfg, w, rank, names, seed, std=0.05):
    rngs = [np.random.default_rng(s) for s in np.random.SeedSequence(seed + 6000003).spawn(2 * len(sb.MATRIX_NAMES))]
    ad = {}
    for i, n in enumerate(sb.MATRIX_NAMES):
        if n not in names:
            continue
        out, inn = w[n].shape
        A = synth.to_storage(rngs[2 * i].standard_normal((rank, inn), dtype=np.float32) * np.float32(std), cfg["dtype"])
        B = synth.to_storage(rngs[2 * i + 1].standard_normal((out, rank), dtype=np.float32) * np.float32(std), cfg["dtype"])
        ad[n] = (A, B)
    return ad


def lora_case(cfg, T, chunk, rank, names=sb.MATRIX_NAMES, batch=1, scale=2.0, seed=0, first=None, tol=None, std=0.05):
    inp = synth.layer_inputs(cfg, seed=seed, seq_len=T, batch=batch)
    ad = make_adapters(cfg, inp["w"], rank, names, seed, std)
    _, dx_ref, dA_ref, dB_ref = o_lora.layer_forward_backward(inp["x"], inp["w"], ad, scale, oracle_cfg(cfg), inp["dy"], first)
    dt = cfg["dtype"]
    w = {k: dev(v, dt) for k, v in inp["w"].items()}
    ad_dev = {n: (dev(A, dt), dev(B, dt)) for n, (A, B) in ad.items()}
    lc = lib_layer_cfg(cfg, T, chunk, batch, seq_first=first)
    dx, da, db = sb.streambp_layer_lora_backward(lc, w, ad_dev, rank, scale, dev(inp["x"], dt), dev(inp["dy"], dt))
    torch.cuda.synchronize()
    tol = tol or TOL[dt]
    assert set(da) == set(names) and set(db) == set(names)
    assert_close(host(dx), dx_ref, tol, "dx")
    for n in names:
        assert da[n].dtype == torch.float32 and tuple(da[n].shape) == ad[n][0].shape
        assert_close(host(da[n]), dA_ref[n], tol, f"dA[{n}]")
        assert_close(host(db[n]), dB_ref[n], tol, f"dB[{n}]")
    return w, ad_dev, lc, inp, (dx, da, db)


@pytest.mark.parametrize("rank", [4, 32])
def test_adapter_gradients_mfma_path(rank):
    lora_case(MID16, 640, 256, rank)
    lora_case(BIG16, 700, 256, rank, batch=2, seed=1)


def test_adapter_gradients_shape_agnostic_paths():
    lora_case(TINY, 96, 40, 3, batch=2, seed=2)
    lora_case(ODD16, 150, 64, 5, seed=3)


def test_attention_only_adapters_and_masks():
    # the common choice: adapters on the query and value projections only; with a sliding window and padding in front
    lora_case(MID16, 500, 128, 8, names=("wq", "wv"), batch=2, seed=4, first=[60, 0])
    lora_case(dict(MID16, window=150), 500, 128, 8, names=("wq", "wv", "wdown"), seed=5)


def test_adapter_gradients_accumulate_and_are_chunk_invariant():
    w, ad, lc, inp, (dx, da, db) = lora_case(MID16, 640, 256, 16, seed=6)
    x, dy = dev(inp["x"], "bf16"), dev(inp["dy"], "bf16")
    da2 = {n: t.clone() for n, t in da.items()}
    db2 = {n: t.clone() for n, t in db.items()}
    sb.streambp_layer_lora_backward(lc, w, ad, 16, 2.0, x, dy, da=da2, db=db2)
    dx_b, da_b, db_b = sb.streambp_layer_lora_backward(lib_layer_cfg(MID16, 640, 128), w, ad, 16, 2.0, x, dy)
    torch.cuda.synchronize()
    for n in da:
        assert_close(host(da2[n]), 2 * host(da[n]), 1e-6, n)                    # +=
        assert_close(host(db2[n]), 2 * host(db[n]), 1e-6, n)
        assert_close(host(da_b[n]), host(da[n]), 1e-2, n)                       # chunk size: rounding order only
        assert_close(host(db_b[n]), host(db[n]), 1e-2, n)


def test_zero_adapters_reproduce_the_plain_layer_bit_for_bit():
    # B = 0: W + s B A = W exactly, so dx must equal the plain entry point's, and dA must be exactly zero
    cfg, T, chunk = MID16, 333, 128
    inp = synth.layer_inputs(cfg, seed=7, seq_len=T)
    ad = make_adapters(cfg, inp["w"], 8, sb.MATRIX_NAMES, 7)
    w = {k: dev(v, "bf16") for k, v in inp["w"].items()}
    ad0 = {n: (dev(A, "bf16"), torch.zeros(B.shape, dtype=torch.bfloat16, device="cuda")) for n, (A, B) in ad.items()}
    x, dy = dev(inp["x"], "bf16"), dev(inp["dy"], "bf16")
    lc = lib_layer_cfg(cfg, T, chunk, dw_group_rows=1)
    dx_plain, _ = sb.streambp_layer_backward(lc, w, x, dy)
    dx, da, db = sb.streambp_layer_lora_backward(lc, w, ad0, 8, 2.0, x, dy)
    torch.cuda.synchronize()
    assert torch.equal(dx, dx_plain)
    assert all(torch.all(t == 0) for t in da.values())
    assert all(float(t.abs().max()) > 0 for t in db.values())


def test_adapter_mode_at_7b_widths_vs_oracle():
    # rank 32 on all seven matrices, 7B widths, the bench's chunk of 2048 rows (T = 2560: one full chunk and a ragged one)
    cfg = synth.CONFIGS["7b"]
    before = sb.streambp_generic_launches()
    # adapter entries N(0, 0.02): the update s B A has a fifth of the base matrices' scale (with N(0, 0.05) it exceeds them and
    # the layer's scores grow until the softmax rows are peaked - the adversarial regime of the large-magnitude test)
    lora_case(cfg, 2560, 2048, 32, seed=8, std=0.02)
    assert sb.streambp_generic_launches() == before
