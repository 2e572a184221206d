"""The attention backward without a workspace (streambp_attn_chunk_backward_noalloc: scratch inside the library's device
image) against the entry point that takes a caller workspace: same kernels, so the results must be bit-identical; two
calls in a row, the second with a smaller chunk, so that stale contents of the shared scratch would show."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2506_03077_amd import binding as sb
from paper_2506_03077_amd import synth

from gpu_util import dev

pytestmark = pytest.mark.gpu


def both_ways(Hq, Hkv, dh, s, c, seed, dtype="bf16"):
    inp = synth.attn_inputs(Hq, Hkv, dh, s, c, dtype, seed)
    q, k, v, d_o = (dev(inp[n], dtype) for n in ("q", "k", "v", "d_o"))
    ac = sb.attn_cfg(sb.SBP_BF16 if dtype == "bf16" else sb.SBP_F32, Hq, Hkv, dh, s, c, 1.0 / np.sqrt(dh))
    o, lse = sb.streambp_attn_chunk_forward(ac, q, k, v)
    dq_a, dk_a, dv_a = sb.streambp_attn_chunk_backward(ac, q, k, v, o, lse, d_o)
    dq_b = torch.full_like(q, float("nan"))
    dk_b = torch.zeros(k.shape, dtype=torch.float32, device="cuda")
    dv_b = torch.zeros(v.shape, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = sb.lib().streambp_attn_chunk_backward_noalloc(C.byref(ac), q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                                       lse.data_ptr(), d_o.data_ptr(), dq_b.data_ptr(), dk_b.data_ptr(),
                                                       dv_b.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == 0, sb.streambp_last_error()
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(dq_a, dq_b) and torch.equal(dk_a, dk_b) and torch.equal(dv_a, dv_b)
    assert bool(torch.isfinite(dq_b.float()).all())


def test_noalloc_backward_matches_the_workspace_entry_point_twice_in_a_row():
    both_ways(8, 2, 128, 700, 333, seed=1)        # MFMA kernels, ragged tiles
    both_ways(8, 2, 128, 64, 40, seed=2)          # a smaller call right after: the scratch still holds the first call's values
    both_ways(4, 2, 16, 10, 20, seed=3, dtype="f32")   # shape-agnostic kernels use the same scratch
