"""Single kernels of the library against numpy (needs an MI355X)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _gemm_case(M, N, K, a_k, b_k, seed, epilogue, arith=0):
    import torch
    from paper_2602_21597_amd import binding
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = rng.standard_normal((K, N)).astype(np.float32)
    want = A.astype(np.float64) @ B.astype(np.float64)
    # what bounds the error of every single output element: the sizes of its own terms
    scale = np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64)
    At = torch.from_numpy(np.ascontiguousarray(A if a_k else A.T)).cuda()      # [M,K] or [K,M]
    Bt = torch.from_numpy(np.ascontiguousarray(B.T if b_k else B)).cuda()      # [N,K] or [K,N]
    kw = {}
    out_rows = None
    if epilogue:
        bias = rng.standard_normal(N).astype(np.float32)
        mask = rng.standard_normal((M, N)).astype(np.float32)
        addend = rng.standard_normal((M, N)).astype(np.float32)
        perm = rng.permutation(M + 5)[:M].astype(np.int32)
        want = np.maximum(want + bias, 0.0)
        want = np.where(mask > 0, want, 0.0) + addend
        scale = scale + np.abs(bias)[None, :] + np.abs(addend)
        full = np.zeros((M + 5, N))
        full[perm] = want
        want = full
        full = np.ones((M + 5, N))             # rows the kernel must leave untouched: exactly zero
        full[perm] = scale
        scale = full
        out_rows = M + 5
        kw = dict(bias=torch.from_numpy(bias).cuda(), relu=True, mask=torch.from_numpy(mask).cuda(),
                  addend=torch.from_numpy(addend).cuda(), dst_row=torch.from_numpy(perm).cuda())
    got = binding.debug_gemm(At, Bt, M, N, K, a_kcontig=a_k, b_kcontig=b_k, out_rows=out_rows, arith=arith,
                             **kw).cpu().numpy()
    # element by element against the sum of |a||b| of that element (an error confined to a few
    # elements of a ragged edge tile cannot hide behind the largest entry of the matrix), and,
    # as before, against the largest entry
    bound = 2e-6 * max(1.0, np.sqrt(K) / 8)
    # (rounding errors of the K accumulation steps are relative to partial sums, which stay far
    # below the sum of the absolute terms: a tenth of the matrix-wide bound)
    worst = (np.abs(got - want) / scale).max()
    assert worst < 0.1 * bound, (M, N, K, a_k, b_k, epilogue, arith, "per element", worst)
    if epilogue:
        untouched = np.ones(M + 5, bool)
        untouched[perm] = False
        assert not np.any(got[untouched]), "rows outside dst_row were written"
    err = np.abs(got - want).max() / np.abs(want).max()
    assert err < bound, (M, N, K, a_k, b_k, epilogue, arith, err)
    return worst


@pytest.mark.parametrize("layout", [(True, True), (True, False), (False, False)])
def test_contraction_kernel_all_layouts_and_tile_paths(layout):
    a_k, b_k = layout
    shapes = [(1, 64, 32), (37, 800, 400), (290, 800, 400), (392, 400, 800), (987, 800, 400),
              (64, 32, 64), (33, 36, 20), (5000, 800, 400), (6100, 800, 400), (130, 400, 1352),
              (2400, 448, 640)]         # (the last: the large tile chosen for a mid-size weight-gradient launch)
    for i, (M, N, K) in enumerate(shapes):
        if not a_k:
            M = (M + 3) // 4 * 4        # the m-contiguous A layout needs M % 4 == 0
        if not b_k:
            N = (N + 3) // 4 * 4
        if a_k or b_k:
            K = (K + 3) // 4 * 4
        print("[case] gemm", M, N, K, layout, flush=True)
        # the arithmetic the training step takes for this layout and size, fp32 matrix
        # instructions, and operands split into bf16 pieces: all to the same bound
        worst = 0.0
        for arith in (0, 1, 2):
            worst = max(worst, _gemm_case(M, N, K, a_k, b_k, seed=i, epilogue=False, arith=arith))
            worst = max(worst, _gemm_case(M, N, K, a_k, b_k, seed=100 + i, epilogue=True, arith=arith))
        print("       worst element error / sum |a||b|: %.2e" % worst, flush=True)


@pytest.mark.parametrize("shape", [(1, 400, 800), (37, 400, 800), (200, 400, 800), (630, 400, 800), (987, 400, 800),
                                   (45, 72, 136), (300, 36, 20), (96, 128, 64)])
def test_mlp_chain_with_operands_as_pieces(shape):
    """Forward and backward launch pairs of one MLP with the weights split once and the hidden rows
    handed on as pieces, against numpy in fp64, element by element against the sum of |a||b|."""
    import torch
    from paper_2602_21597_amd import binding
    M, d, h = shape
    rng = np.random.default_rng(M + d)
    X = rng.standard_normal((M, d)).astype(np.float32)
    W1 = (rng.standard_normal((h, d)) / np.sqrt(d)).astype(np.float32)
    W2 = (rng.standard_normal((d, h)) / np.sqrt(h)).astype(np.float32)
    b1 = rng.standard_normal(h).astype(np.float32)
    b2 = rng.standard_normal(d).astype(np.float32)
    mask = rng.standard_normal((M, h)).astype(np.float32)
    f = lambda a: torch.from_numpy(a).cuda()
    X64, W164, W264 = X.astype(np.float64), W1.astype(np.float64), W2.astype(np.float64)
    bar = 0.1 * 2e-6 * max(1.0, np.sqrt(max(d, h)) / 8)
    for backward in (False, True):
        print("[case] mlp chain", shape, "backward" if backward else "forward", flush=True)
        H, Y, used = binding.debug_mlp(f(X), f(W1), f(b1), f(W2), f(b2), mask=f(mask), backward=backward)
        H, Y = H.cpu().numpy(), Y.cpu().numpy()
        assert used & 1, "the weights were not read as pieces"
        small = ((M + 31) // 32) * ((h + 63) // 64) * 2 <= 512
        assert bool(used & 2) == small, ("hidden rows as pieces", used, small)
        if not backward:
            pre = X64 @ W164.T + b1
            wantH = np.maximum(pre, 0.0)
            scaleH = np.abs(X64) @ np.abs(W164.T) + np.abs(b1)
            # a hidden value rounded to zero or not at a pre-activation within rounding of zero: either is right
            free = np.abs(pre) < bar * scaleH
            W2x, scale2 = W264.T, np.abs(W264.T)
            add = b2
        else:
            wantH = np.where(mask > 0, X64 @ W264, 0.0)
            scaleH = np.abs(X64) @ np.abs(W264)
            free = np.zeros_like(wantH, bool)
            W2x, scale2 = W164, np.abs(W164)
            add = 0.0
        errH = np.abs(H - wantH) / scaleH
        assert errH[~free].max() < bar, ("H", shape, backward, errH[~free].max())
        # the second launch against the first one's own (fp32) output: its operand, whichever form it took
        wantY = H.astype(np.float64) @ W2x + add
        scaleY = np.abs(H).astype(np.float64) @ scale2 + np.abs(add)
        errY = (np.abs(Y - wantY) / np.maximum(scaleY, 1e-30)).max()
        assert errY < bar, ("Y", shape, backward, errY)
        print("       worst element error / sum |a||b|: H %.2e  Y %.2e  (pieces of H: %s)" % (errH[~free].max(), errY, bool(used & 2)), flush=True)


def test_split_contraction_keeps_fp32_accuracy_where_bf16_alone_would_not():
    """Operands with a wide spread of magnitudes and with values that need all 24 significand
    bits: the split arithmetic must stay at the fp32 level (a single bf16 piece would be off
    by 2^-9, two pieces by 2^-17)."""
    import torch
    from paper_2602_21597_amd import binding
    rng = np.random.default_rng(7)
    M, N, K = 96, 160, 528
    A = (rng.standard_normal((M, K)) * np.exp2(rng.integers(-12, 12, (M, K)))).astype(np.float32)
    B = (1.0 + rng.random((K, N)) * 2.0 ** -12).astype(np.float32)          # differ only in the low bits
    want = A.astype(np.float64) @ B.astype(np.float64)
    scale = np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64)     # no cancellation credit
    for arith in (1, 2):
        got = binding.debug_gemm(torch.from_numpy(A).cuda(), torch.from_numpy(np.ascontiguousarray(B.T)).cuda(),
                                 M, N, K, arith=arith).cpu().numpy()
        err = (np.abs(got - want) / scale).max()
        print("[case] arith", arith, "error relative to sum |a||b|:", err, flush=True)
        assert err < 2e-6, (arith, err)
