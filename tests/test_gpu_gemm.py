"""GPU unit tests of the GEMM dispatcher (MFMA kernel and shape-agnostic kernel)
against numpy fp64 products of the same bf16-rounded inputs.  The closed form
of the paper's linear example (App. A.1) is checked too: with L = sum(Z),
dW2 = Y^T 1 and dW1 = X^T (1 W2^T), accumulated chunk by chunk."""
import numpy as np
import pytest
import torch

from paper_2506_03077_amd import binding as sb
from paper_2506_03077_amd import synth

from gpu_util import assert_close, dev, host

pytestmark = pytest.mark.gpu


def run(M, N, K, ta, tb, out="f32", acc=False, seed=0, expect_mfma=None, dtype="bf16"):
    rng = np.random.default_rng(seed)
    A = synth.to_storage(rng.normal(size=(K, M) if ta else (M, K)), dtype)
    B = synth.to_storage(rng.normal(size=(N, K) if tb else (K, N)), dtype)
    C0 = synth.to_storage(rng.normal(size=(M, N)), out) if acc else np.zeros((M, N), np.float32)
    opA = A.T.astype(np.float64) if ta else A.astype(np.float64)
    opB = B.T.astype(np.float64) if tb else B.astype(np.float64)
    want = opA @ opB + C0
    Cd = dev(C0, out) if acc else torch.full((M, N), float("nan"), device="cuda",
                                            dtype=torch.bfloat16 if out == "bf16" else torch.float32)
    scratch = torch.empty(8 * M * N, dtype=torch.float32, device="cuda")
    used = sb.debug_gemm(dev(A, dtype), dev(B, dtype), Cd, M, N, K, ta, tb, acc, scratch)
    torch.cuda.synchronize()
    if expect_mfma is not None:
        assert used == int(expect_mfma), f"kernel selection: used_mfma={used}"
    assert_close(host(Cd), want, 4e-3 if out == "bf16" else 2e-5, f"C M={M} N={N} K={K} ta={ta} tb={tb}")


LAYOUTS = [(False, True), (False, False), (True, False)]      # NT, NN, TN


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_mfma_one_tile(ta, tb):
    run(256, 256, 256, ta, tb, expect_mfma=True)


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_mfma_several_tiles_all_outputs(ta, tb):
    run(512, 768, 320 if ta else 384, ta, tb, out="f32", expect_mfma=True)
    run(512, 768, 384, ta, tb, out="bf16", expect_mfma=True, seed=1)
    run(512, 768, 384, ta, tb, out="f32", acc=True, expect_mfma=True, seed=2)


@pytest.mark.parametrize("M", [1, 37, 255, 257, 300, 700])
def test_mfma_ragged_rows(M):
    run(M, 512, 128, False, True, expect_mfma=True)
    run(M, 256, 192, False, False, out="bf16", expect_mfma=True)


@pytest.mark.parametrize("K", [1, 63, 65, 100, 333, 1000])
def test_mfma_ragged_reduction_in_dw_form(K):
    run(256, 512, K, True, False, acc=True, expect_mfma=True)


def test_mfma_split_k_paths():
    run(256, 256, 8192, False, True, expect_mfma=True)               # 1 tile, long K -> split
    run(300, 512, 4096, False, False, out="bf16", expect_mfma=True)
    run(512, 256, 4096, False, False, acc=True, expect_mfma=True)
    run(256, 256, 4000, True, False, acc=True, expect_mfma=True)     # ragged split


def test_mfma_split_k_eight_ways_and_unaligned_groups():
    run(256, 512, 8192, False, True, expect_mfma=True)                # 2 tiles, 128 K steps: 8 slices, one per XCD
    run(256, 768, 8192, False, False, out="bf16", expect_mfma=True)   # 3 tiles x 8 slices
    run(256, 768, 3072, False, False, expect_mfma=True, seed=3)       # 4 slices, 3 tiles: not a multiple of the XCD group
    run(200, 1280, 2048, False, True, acc=True, expect_mfma=True, seed=4)   # ragged rows, 5 tiles x 4 slices


def test_two_operand_pairs_in_one_launch():
    # C = A B + A2 B2 (the shape of dm = dgate W_g + dup W_u): the two products are the two slices of one split-K launch;
    # where that does not fit (no scratch, odd shapes) the dispatcher runs them one after the other
    rng = np.random.default_rng(12)
    for (M, N, K, scratch_ok, expect) in ((300, 512, 1024, True, 1), (300, 512, 1024, False, 1), (70, 45, 33, True, 0)):
        A, A2 = (synth.to_storage(rng.normal(size=(M, K)), "bf16") for _ in range(2))
        B, B2 = (synth.to_storage(rng.normal(size=(K, N)), "bf16") for _ in range(2))
        want = A.astype(np.float64) @ B.astype(np.float64) + A2.astype(np.float64) @ B2.astype(np.float64)
        C = torch.full((M, N), float("nan"), device="cuda", dtype=torch.float32)
        scratch = torch.empty(2 * M * N, dtype=torch.float32, device="cuda") if scratch_ok else None
        used = sb.debug_gemm(dev(A, "bf16"), dev(B, "bf16"), C, M, N, K, False, False, False, scratch,
                             A2=dev(A2, "bf16"), B2=dev(B2, "bf16"))
        torch.cuda.synchronize()
        assert used == expect
        assert_close(host(C), want, 2e-5, f"pair M={M} N={N} K={K} scratch={scratch_ok}")


def test_row_statistics_from_the_store_epilogue():
    # C = A B^T with fp32 C, plus per row and block of 256 columns the pair (max, sum of exp(c - max)) that the LM head's
    # log-sum-exp is merged from: the maxima are those of the stored C bit for bit, the sums follow to fp32 rounding,
    # rows beyond M are never written; a problem the MFMA kernel cannot take refuses the request instead of ignoring it
    rng = np.random.default_rng(21)
    for (M, N, K, scale) in ((256, 256, 64, 1.0), (300, 1024, 192, 1.0), (37, 512, 128, 8.0)):
        A = synth.to_storage(rng.normal(size=(M, K)) * scale, "bf16")
        B = synth.to_storage(rng.normal(size=(N, K)), "bf16")
        C = torch.full((M, N), float("nan"), device="cuda", dtype=torch.float32)
        nb = N // 256
        stats = torch.full((M + 3, nb, 2), -7.0, device="cuda", dtype=torch.float32)
        used = sb.debug_gemm(dev(A, "bf16"), dev(B, "bf16"), C, M, N, K, False, True, row_stats=stats)
        torch.cuda.synchronize()
        assert used == 1
        want = A.astype(np.float64) @ B.astype(np.float64).T
        assert_close(host(C), want, 2e-5, f"C M={M} N={N} K={K}")
        Cb = C.cpu().numpy().reshape(M, nb, 256)
        st = stats.cpu().numpy()
        assert np.array_equal(st[:M, :, 0], Cb.max(axis=2)), "block maxima differ from the stored C"
        se = np.exp(Cb.astype(np.float64) - Cb.max(axis=2, keepdims=True)).sum(axis=2)
        assert np.allclose(st[:M, :, 1], se, rtol=2e-5, atol=0), np.abs(st[:M, :, 1] / se - 1).max()   # 256 fp32 terms
        assert np.all(st[M:] == -7.0), "statistics written past the last row"
    A = torch.zeros((64, 96), device="cuda", dtype=torch.bfloat16)
    B = torch.zeros((100, 96), device="cuda", dtype=torch.bfloat16)
    with pytest.raises(sb.StreamBPError):
        sb.debug_gemm(A, B, torch.zeros((64, 100), device="cuda"), 64, 100, 96, False, True,
                      row_stats=torch.zeros((64, 1, 2), device="cuda"))


def test_mfma_segmented_weight_gradient():
    # C += sum_s A_s^T B_s in one launch; segments of different length, two of them cut short by a device row count
    rng = np.random.default_rng(5)
    M, N, Ks, limits = 512, 256, (300, 1000, 64, 128, 192, 77, 256, 500), (250, None, 0, None, None, 70, None, 499)
    As = [synth.to_storage(rng.normal(size=(K, M)), "bf16") for K in Ks]
    Bs = [synth.to_storage(rng.normal(size=(K, N)), "bf16") for K in Ks]
    C0 = rng.normal(size=(M, N)).astype(np.float32)
    want = C0.astype(np.float64)
    for A, B, K, lim in zip(As, Bs, Ks, limits):
        k = K if lim is None else lim
        want = want + A[:k].T.astype(np.float64) @ B[:k].astype(np.float64)
    for n in (2, 4, 7, 8):
        Cd = dev(C0, "f32")
        rows = [None if lim is None else torch.tensor([lim], dtype=torch.int32, device="cuda") for lim in limits[:n]]
        used = sb.debug_gemm_dw_segments([dev(a, "bf16") for a in As[:n]], [dev(b, "bf16") for b in Bs[:n]], Cd, M, N, Ks[:n], rows)
        torch.cuda.synchronize()
        assert used == 1
        part = C0.astype(np.float64)
        for A, B, K, lim in list(zip(As, Bs, Ks, limits))[:n]:
            k = K if lim is None else lim
            part = part + A[:k].T.astype(np.float64) @ B[:k].astype(np.float64)
        assert_close(host(Cd), part, 2e-5, f"segmented dW, {n} segments")
    assert part.shape == want.shape


def test_weight_gradient_into_bf16_accumulator():
    # C (bf16) += A^T B: read, add in fp32, round once
    run(512, 768, 320, True, False, out="bf16", acc=True, expect_mfma=True, seed=6)     # one launch, ragged reduction
    run(512, 256, 2048, True, False, out="bf16", acc=True, expect_mfma=True, seed=7)    # split-K, reduced into the bf16 C
    run(130, 172, 64, True, False, out="bf16", acc=True, expect_mfma=False, seed=8)     # shape-agnostic kernel
    rng = np.random.default_rng(9)
    M, N, Ks = 512, 256, (300, 200)
    As = [synth.to_storage(rng.normal(size=(K, M)), "bf16") for K in Ks]
    Bs = [synth.to_storage(rng.normal(size=(K, N)), "bf16") for K in Ks]
    C0 = synth.to_storage(rng.normal(size=(M, N)), "bf16")
    want = C0.astype(np.float64) + sum(A.T.astype(np.float64) @ B.astype(np.float64) for A, B in zip(As, Bs))
    Cd = dev(C0, "bf16")
    used = sb.debug_gemm_dw_segments([dev(a, "bf16") for a in As], [dev(b, "bf16") for b in Bs], Cd, M, N, Ks)
    torch.cuda.synchronize()
    assert used == 1
    assert_close(host(Cd), want, 4e-3, "segmented dW into bf16")


def run_wide(M, N, K, ta, tb, out="f32", acc=False, seed=0, pad=24):
    """Like run(), with C a column slice of a wider buffer: the columns past N must come back untouched."""
    rng = np.random.default_rng(seed)
    A = synth.to_storage(rng.normal(size=(K, M) if ta else (M, K)), "bf16")
    B = synth.to_storage(rng.normal(size=(N, K) if tb else (K, N)), "bf16")
    C0 = synth.to_storage(rng.normal(size=(M, N)), out) if acc else np.zeros((M, N), np.float32)
    want = (A.T if ta else A).astype(np.float64) @ (B.T if tb else B).astype(np.float64) + C0
    tdt = torch.bfloat16 if out == "bf16" else torch.float32
    full = torch.full((M, N + pad), -7.0, device="cuda", dtype=tdt)
    if acc:
        full[:, :N] = dev(C0, out)
    scratch = torch.empty(8 * M * N, dtype=torch.float32, device="cuda")
    used = sb.debug_gemm(dev(A, "bf16"), dev(B, "bf16"), full[:, :N], M, N, K, ta, tb, acc, scratch)
    torch.cuda.synchronize()
    assert used == 1, "the MFMA kernel must take ragged output widths"
    assert torch.all(full[:, N:] == -7.0), "written past the last column"
    assert_close(host(full[:, :N]), want, 4e-3 if out == "bf16" else 2e-5, f"C M={M} N={N} K={K} ta={ta} tb={tb} out={out} acc={acc}")


@pytest.mark.parametrize("ta,tb", LAYOUTS)
@pytest.mark.parametrize("N", [8, 128, 264, 648])
def test_mfma_ragged_output_width(ta, tb, N):
    # output widths that are multiples of 8 but not of the 256-wide tile (a 151936-word vocabulary is 593.5 tiles): the
    # last column tile clamps its loads and masks its stores; in the weight-gradient form the rows are ragged too
    M = 264 if ta else 300
    K = 200 if ta else 192
    run_wide(M, N, K, ta, tb, out="f32", seed=N)
    run_wide(M, N, K, ta, tb, out="bf16", seed=N + 1)
    run_wide(M, N, K, ta, tb, out="f32", acc=True, seed=N + 2)
    if ta:
        run_wide(M, N, K, ta, tb, out="bf16", acc=True, seed=N + 3)
        run_wide(8, N, 100, ta, tb, out="f32", acc=True, seed=N + 4)          # eight rows of a ragged weight gradient


def test_mfma_ragged_output_width_split_k_pairs_and_segments():
    run_wide(256, 264, 8192, False, True, seed=31)                     # two column tiles, the second 8 wide, eight K slices
    run_wide(300, 392, 4096, False, False, out="bf16", seed=32)
    run_wide(264, 392, 4000, True, False, acc=True, seed=33)
    rng = np.random.default_rng(34)
    M, N, Ks = 520, 392, (300, 200, 77)                                # segmented weight gradient, ragged in both directions
    As = [synth.to_storage(rng.normal(size=(K, M)), "bf16") for K in Ks]
    Bs = [synth.to_storage(rng.normal(size=(K, N)), "bf16") for K in Ks]
    for out in ("f32", "bf16"):
        C0 = synth.to_storage(rng.normal(size=(M, N)), out)
        want = C0.astype(np.float64) + sum(A.T.astype(np.float64) @ B.astype(np.float64) for A, B in zip(As, Bs))
        Cd = dev(C0, out)
        used = sb.debug_gemm_dw_segments([dev(a, "bf16") for a in As], [dev(b, "bf16") for b in Bs], Cd, M, N, Ks)
        torch.cuda.synchronize()
        assert used == 1
        assert_close(host(Cd), want, 4e-3 if out == "bf16" else 2e-5, f"ragged segmented dW into {out}")


def test_row_statistics_with_a_ragged_last_column_block():
    rng = np.random.default_rng(35)
    for (M, N, K) in ((300, 648, 192), (64, 8, 64), (257, 1400, 128)):
        A = synth.to_storage(rng.normal(size=(M, K)) * 3.0, "bf16")
        B = synth.to_storage(rng.normal(size=(N, K)), "bf16")
        nb = -(-N // 256)
        full = torch.full((M, N + 40), -7.0, device="cuda", dtype=torch.float32)
        stats = torch.full((M + 3, nb, 2), -7.0, device="cuda", dtype=torch.float32)
        used = sb.debug_gemm(dev(A, "bf16"), dev(B, "bf16"), full[:, :N], M, N, K, False, True, row_stats=stats)
        torch.cuda.synchronize()
        assert used == 1 and torch.all(full[:, N:] == -7.0) and torch.all(stats[M:] == -7.0)
        C = full[:, :N].cpu().numpy()
        assert_close(C, A.astype(np.float64) @ B.astype(np.float64).T, 2e-5, f"C M={M} N={N}")
        st = stats.cpu().numpy()
        for b in range(nb):
            blk = C[:, b * 256:min(N, (b + 1) * 256)]
            assert np.array_equal(st[:M, b, 0], blk.max(axis=1)), f"block {b}: maxima differ from the stored C"
            se = np.exp(blk.astype(np.float64) - blk.max(axis=1, keepdims=True)).sum(axis=1)
            assert np.allclose(st[:M, b, 1], se, rtol=2e-5, atol=0)


def test_mfma_bigger_square():
    run(1024, 1024, 1024, False, True, out="bf16", expect_mfma=True)


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_generic_odd_shapes(ta, tb):
    run(70, 45, 33, ta, tb, expect_mfma=False)
    run(70, 45, 33, ta, tb, out="bf16", expect_mfma=False)
    run(130, 172, 64, ta, tb, acc=True, expect_mfma=False, dtype="f32")


def test_linear_example_closed_form():
    # Y = X W1, Z = Y W2, L = sum(Z): dZ = 1, dY = 1 W2^T, dW1 = X^T dY, dW2 = Y^T 1 (App. A.1),
    # accumulated over D chunks of rows with the dW-form GEMM (C += A^T B).
    rng = np.random.default_rng(0)
    D, rows, m, n, k = 3, 200, 256, 512, 256
    X = synth.to_storage(rng.normal(size=(D * rows, m)), "bf16")
    W1 = synth.to_storage(rng.normal(size=(m, n)) * 0.05, "bf16")
    W2 = synth.to_storage(rng.normal(size=(n, k)) * 0.05, "bf16")
    ones = torch.ones((rows, k), dtype=torch.bfloat16, device="cuda")
    dW1 = torch.zeros((m, n), dtype=torch.float32, device="cuda")
    dW2 = torch.zeros((n, k), dtype=torch.float32, device="cuda")
    W1d, W2d = dev(W1, "bf16"), dev(W2, "bf16")
    Ys = []
    for i in range(D):
        Xi = dev(X[i * rows:(i + 1) * rows], "bf16")
        Yi = torch.empty((rows, n), dtype=torch.bfloat16, device="cuda")
        sb.debug_gemm(Xi, W1d, Yi, rows, n, m, False, False)               # Y_i = X_i W1
        dYi = torch.empty((rows, n), dtype=torch.bfloat16, device="cuda")
        sb.debug_gemm(ones, W2d, dYi, rows, n, k, False, True)             # dY_i = 1 W2^T
        sb.debug_gemm(Xi, dYi, dW1, m, n, rows, True, False, acc=True)     # dW1 += X_i^T dY_i
        sb.debug_gemm(Yi, ones, dW2, n, k, rows, True, False, acc=True)    # dW2 += Y_i^T 1
        Ys.append(host(Yi))
    torch.cuda.synchronize()
    X64, W164, W264 = X.astype(np.float64), W1.astype(np.float64), W2.astype(np.float64)
    want_dW1 = np.outer(X64.sum(axis=0), W264.sum(axis=1))                 # X^T (1 W2^T) in closed form
    want_dW2 = np.repeat((X64 @ W164).sum(axis=0)[:, None], k, axis=1)     # Y^T 1
    assert_close(host(dW1), want_dW1, 5e-3, "dW1")
    assert_close(host(dW2), want_dW2, 5e-3, "dW2")


def test_mfma_rate_probe_counts_what_it_claims():
    # the benchmark's pure-MFMA probe: with all-one fragments every accumulator element grows by 16 per product, so each
    # thread's sum over its 8 x 16 accumulator registers after n rounds is exactly 8 * 16 * 16 * n (the flop count it is
    # credited with: 2 * 32*32*16 * 8 products per wave and round)
    ones = torch.ones(32768, dtype=torch.bfloat16, device="cuda")
    sink = torch.full((4 * 512,), -1.0, dtype=torch.float32, device="cuda")
    for n, reads in ((0, 0), (1, 0), (37, 0), (37, 6), (37, 8)):     # fragments re-read from LDS hold the same ones
        rc = sb.lib().streambp_debug_mfma_rate(ones.data_ptr(), sink.data_ptr(), 4, n, reads, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert rc == 0
        assert torch.all(sink == 8 * 16 * 16 * n), (n, reads)
    assert sb.lib().streambp_debug_mfma_rate(None, sink.data_ptr(), 4, 1, 0, None) == -1
    assert sb.lib().streambp_debug_mfma_rate(ones.data_ptr(), sink.data_ptr(), 4, 1, 5, None) == -2
    assert sb.debug_mfma_rate(ones, workgroups=64, iters=100, repeats=1) > 0
    assert sb.debug_mfma_rate(ones, workgroups=64, iters=100, repeats=1, lds_reads=8) > 0


def test_softmax_numerators_from_the_store_epilogue():
    # The LM head's fused store (Sec. 5 names fused backward operators as future work): instead of the fp32 logits c the GEMM
    # leaves E = exp(c - max of the row's 256-column block) in bf16, the block's (max, sum) pair and the fp32 logit of each
    # row's target column.  Against fp64 products of the same bf16 inputs: the maxima and target logits to fp32 GEMM
    # rounding, the sums likewise (they are taken from the unrounded exponentials), E to one bf16 rounding; a ragged last
    # column block (N = 1416 = 5.53 blocks), ragged rows, a row-index indirection, targets outside [0, N) (entry untouched),
    # and nothing written past row M.
    rng = np.random.default_rng(31)
    for (M, N, K, scale, indirect) in ((256, 256, 64, 1.0, False), (300, 1416, 192, 1.0, True), (37, 512, 128, 6.0, False)):
        A = synth.to_storage(rng.normal(size=(M, K)) * scale, "bf16")
        B = synth.to_storage(rng.normal(size=(N, K)), "bf16")
        nb = (N + 255) // 256
        n_src = M + 50
        perm = rng.permutation(n_src)[:M].astype(np.int32) if indirect else None
        tg_src = rng.integers(0, N, size=n_src if indirect else M).astype(np.int32)
        tg_src[rng.integers(0, len(tg_src), size=3)] = [-1, N, N + 7]           # never used as an index
        tgt = tg_src[perm] if indirect else tg_src
        E = torch.full((M + 2, N), 3.0, device="cuda", dtype=torch.bfloat16)
        stats = torch.full((M + 3, nb, 2), -7.0, device="cuda", dtype=torch.float32)
        zt = torch.full((M + 3,), -5.0, device="cuda", dtype=torch.float32)
        used = sb.debug_gemm_numerators(dev(A, "bf16"), dev(B, "bf16"), E[:M], stats, torch.from_numpy(tg_src).cuda(), zt,
                                        row_index=None if perm is None else torch.from_numpy(perm).cuda())
        torch.cuda.synchronize()
        assert used == 1
        c = A.astype(np.float64) @ B.astype(np.float64).T
        cpad = np.full((M, nb * 256), -np.inf)
        cpad[:, :N] = c
        blocks = cpad.reshape(M, nb, 256)
        bmax = blocks.max(axis=2)
        bsum = np.exp(blocks - bmax[:, :, None]).sum(axis=2)
        st = stats.cpu().numpy()
        tol_c = 2e-5 * np.abs(c).max()
        assert np.abs(st[:M, :, 0] - bmax).max() <= tol_c
        assert np.allclose(st[:M, :, 1], bsum, rtol=1e-4 + 2 * tol_c, atol=0), np.abs(st[:M, :, 1] / bsum - 1).max()
        assert np.all(st[M:] == -7.0), "statistics written past the last row"
        want_e = np.exp(blocks - bmax[:, :, None]).reshape(M, nb * 256)[:, :N]
        got_e = E[:M].float().cpu().numpy()
        assert np.all(np.abs(got_e - want_e) <= 2.0 ** -8 * want_e + 2 * tol_c * want_e + 1e-30), np.abs(got_e - want_e).max()
        assert torch.all(E[M:] == 3.0), "E written past the last row"
        valid = (tgt >= 0) & (tgt < N)
        got_zt = zt.cpu().numpy()
        assert np.abs(got_zt[:M][valid] - c[np.arange(M)[valid], tgt[valid]]).max() <= tol_c
        assert np.all(got_zt[:M][~valid] == -5.0) and np.all(got_zt[M:] == -5.0)
    # a problem the MFMA kernel cannot take is refused (nothing written)
    A = torch.zeros((64, 96), device="cuda", dtype=torch.bfloat16)
    B = torch.zeros((104, 96), device="cuda", dtype=torch.bfloat16)
    assert sb.debug_gemm_numerators(A, B, torch.zeros((64, 104), device="cuda", dtype=torch.bfloat16), torch.zeros((64, 1, 2), device="cuda"),
                                    torch.zeros(64, dtype=torch.int32, device="cuda"), torch.zeros(64, device="cuda")) == 0
