"""Helpers for the GPU parity tests: upload a problem, call the C ABI through the binding, and compare an
output with the CPU oracle (whole-output and per-tile-row Frobenius error, and a derived per-element bound)."""
import sys
import time

import numpy as np

TOL = 2e-3          # stated acceptance bound: relative Frobenius error against the float64 oracle
U16 = 2.0 ** -11    # unit roundoff of fp16 (round to nearest)
U32 = 2.0 ** -24    # unit roundoff of fp32
FLOOR16 = 2.0 ** -25  # half the spacing of fp16 denormals: absolute rounding error below 2^-14


def device_problem(p, device="cuda:0"):
    import torch
    import paper_2602_01027_amd as S

    L, s2, s3, s4, index = S.sfmp_pack(p.codes, p.bitmap)
    S.sfmp_layout_set_quant(L, p.group, p.scale_format)
    dp = S.upload_packed(L, s2, s3, s4, index, p.scales, p.zeros, p.bitmap, device)
    cp = torch.from_numpy(p.col_perm).to(device) if p.col_perm is not None else None
    rp = torch.from_numpy(p.row_perm).to(device) if p.row_perm is not None else None
    return dp, cp, rp


def make_workspace(layout, M, device="cuda:0", fill=0xFF):
    """A workspace of the size the library asks for, filled with 0xFF bytes (fp16 / fp32 NaN patterns): the
    library promises that the contents on entry are irrelevant, so the tests hand it the worst contents."""
    import torch
    import paper_2602_01027_amd as S

    nbytes = S.sfmp_gemm_workspace(layout, M)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    ws.fill_(fill)
    return ws


def run_gemm(p, dp=None, cp=None, rp=None, ws=None, X=None, device="cuda:0"):
    """Y (numpy fp16 [M, N]) of the HIP path for problem p."""
    import torch
    import paper_2602_01027_amd as S

    if dp is None:
        dp, cp, rp = device_problem(p, device)
    Xh = p.X if X is None else X
    M = Xh.shape[0]
    Xd = torch.from_numpy(np.ascontiguousarray(Xh)).to(device)
    if ws is None:
        ws = make_workspace(dp.layout, M, device)
    Y = torch.full((M, p.N), float("nan"), dtype=torch.float16, device=device)
    S.sfmp_gemm(Xd, cp, dp.layout, dp.s2, dp.s3, dp.s4, dp.index, dp.scales, dp.zeros, dp.bitmap, rp, Y, ws)
    torch.cuda.synchronize()
    return Y.cpu().numpy()


# ---------------------------------------------------------------------------------------------
# comparison with the oracle
# ---------------------------------------------------------------------------------------------
def mfma_alignment_loss(Xp):
    """V [m, K/64]: per activation row and half tile column, the bits that v_mfma_f32_16x16x32_f16 can drop from the
    products of the decode kernels, in units of the scale (multiply by |s| of the column half's group).

    The decode kernels feed the codes to the matrix cores as fp16 denormals q * 2^(p-24) (p = position of the code's
    field, >= 0).  The instruction aligns its products to a common exponent before it adds them, and it takes the
    NOMINAL exponent of an operand for that - 2^-14 for a denormal, whatever its leading bit - so that the significant
    bits of x_k q 2^(p-24), which reach down to 2^(e_k - 34 + p), can fall below the 24 bits it keeps under the largest
    nominal product exponent E - 14 (E = the largest exponent among the 32 activations of the instruction, one k-step
    of 32 columns).  Measured and pinned by tests/test_gpu_parity.py::test_mfma_alignment_model: a product loses less
    than 2^(E - 38), and only if e_k <= E - 4; the bits are cut off, not rounded (within the 8 products of one lane the
    cut is exactly at 2^(E_lane - 38)).  After the kernel's factors 2^24 2^-p |s| that is less than |s| 2^(E - 14) per
    such product (p = 0 is the worst case).  Returned: per 64 columns, the sum over its two k-steps of 2^(E - 14) x
    (the number of non-zero x_k of the k-step with e_k <= E - 4)."""
    m, K = Xp.shape
    ax = np.abs(Xp).reshape(m, K // 32, 32)
    _, e = np.frexp(ax)                        # |x| = f 2^e with f in [0.5, 1): exponent e - 1
    e = np.maximum(e - 1, -14)                 # (an fp16 denormal counts as 2^-14)
    E = np.where(ax > 0, e, -100).max(axis=2)  # [m, k-steps]; a k-step of zeros loses nothing
    lossy = ((ax > 0) & (e <= E[:, :, None] - 4)).sum(axis=2)
    per_step = np.where(E > -100, np.ldexp(1.0, np.maximum(E, -100) - 14), 0.0) * lossy
    return per_step.reshape(m, K // 64, 2).sum(axis=2)


def elementwise_tolerance(M, K, ref, A, B, X1, T=0.0):
    """Bound on |y_gpu - ref| for one output, from the arithmetic of the kernels (first-order rounding analysis
    with the standard gamma_n = n u / (1 - n u); nothing here is fitted to observed errors).

    ref = sum_j x_j w_j (float64), A = sum_j |x_j| |w_j|, B = sum_j |x_j| (|s| q_j + |z|) >= A, X1 = sum_j |x_j|,
    T = what the matrix instruction's alignment of denormal operands can drop (mfma_alignment_loss times |s|; decode
    kernels only).

    Every path ends in one fp32 -> fp16 rounding of its fp32 sum: u16 |sum| + 2^-25.

    Decode kernels (M <= 16, and chunks of 16 rows of a medium batch): products x * q are exact (11-bit by 4-bit
    significands); per 128-column group they form t = sum x q and sum x in fp32, then acc_q += s t, acc_z += z sum x,
    y = 2^24 acc_q + acc_z, summed over the wavefronts.  The longest chain of fp32 roundings a term passes through:
    at most 4 matrix instructions of 32 products into one accumulator (128), the combination of the field
    positions (3), one fused multiply-add per item of a wavefront and slab (at most ceil(K / 1024)), the final
    combination (1), the sum over 16 wavefronts (16); a product inside a matrix instruction is cut off rather than
    rounded (up to a whole unit in the last place: counted twice): D = 276 + ceil(K / 1024) roundings, each relative
    to a partial sum bounded by B.  Hence |err| <= u16 |ref| + 2^-25 + (1 + u16) (gamma_D B + T).

    MFMA prefill kernel (M > 16): w_j is rounded to fp16 once (|delta_j| <= u16 |w_j| + 2^-25; with bf16
    parameters s q + z is formed in fp32 first: one more u32), products are exact in fp32, and all K products of
    an output go through one accumulator chain (K / 32 matrix instructions of 32 products, each product cut off rather
    than rounded: counted twice; a split K only shortens it):
    |err| <= u16 |ref| + 2^-25 + (1 + u16) ((u16 + u32 + gamma_{2K+8}) A + 2^-25 X1).
    For M > 16 the library chooses between the two paths, so the larger bound applies.
    """
    # (the matrix instruction cuts its aligned products off instead of rounding them - pinned by
    # test_mfma_alignment_model - so each of its products counts as two roundings)
    D = 2 * 128 + 20 + -(-K // 1024)
    g_d = D * U32 / (1.0 - D * U32)
    tol = U16 * np.abs(ref) + FLOOR16 + (1.0 + U16) * (g_d * B + T)
    if M > 16:
        n = 2 * K + 8
        g_k = n * U32 / (1.0 - n * U32)
        tol_pre = U16 * np.abs(ref) + FLOOR16 + (1.0 + U16) * ((U16 + U32 + g_k) * A + FLOOR16 * X1)
        tol = np.maximum(tol, tol_pre)
    return tol


def check_against_oracle(p, Y, feature_rows=None, m_rows=None, block=1024, elementwise=True):
    """Compare Y (fp16 [M, N], columns in original order when p.row_perm is given) with the oracle.

    Asserts (1) relative Frobenius error <= 2e-3 over everything compared, (2) the same bound for every tile row
    on its own (128 output features x the compared activation rows; only when whole tile rows are compared: one
    wrong 16-row slab of one tile cannot hide in the norm of a large matrix), (3) the derived per-element bound of
    `elementwise_tolerance`.  feature_rows: reordered output features to compare (default all, walked in blocks so
    that the float64 dequantised weights of a 70B matrix never exist at once); m_rows: activation rows to compare
    (default all); elementwise=False leaves (3) out (for a kernel with other arithmetic than the bound describes).
    Returns the overall relative Frobenius error."""
    from oracle import sfmp_oracle as O

    Y = np.asarray(Y)
    M, N, K = p.X.shape[0], p.N, p.K
    assert Y.shape == (M, N)
    assert np.isfinite(Y.astype(np.float32)).all()
    mr = np.arange(M) if m_rows is None else np.unique(np.asarray(m_rows, dtype=np.int64))
    X = np.ascontiguousarray(p.X[mr])
    Xabs = np.abs(O.permute_activation(X, p.col_perm))
    X1 = Xabs.sum(axis=1)[:, None]
    whole_tile_rows = feature_rows is None
    feats = np.arange(N, dtype=np.int64) if feature_rows is None else np.unique(np.asarray(feature_rows, dtype=np.int64))
    sabs, zabs = np.abs(p.scales), np.abs(p.zeros)
    V64 = mfma_alignment_loss(O.permute_activation(X, p.col_perm).astype(np.float64))   # [m, K/64]
    half_group = (np.arange(K // 64) * 64) // p.group                                   # parameter row of each column half
    num = den = 0.0
    worst = (0.0, None)
    last_note = time.monotonic()
    for i0 in range(0, feats.size, block):
        if time.monotonic() - last_note > 30.0:  # a long comparison says that it is alive
            print(f"  oracle comparison: feature {i0} of {feats.size}", file=sys.stderr, flush=True)
            last_note = time.monotonic()
        rows = feats[i0:i0 + block]
        ref = O.gemm_rows(X, p.col_perm, p.codes, p.scales, p.zeros, rows)          # [m, rows], reordered features
        A = Xabs @ np.abs(O.dequant_rows(p.codes, p.scales, p.zeros, rows)).T
        B = Xabs @ O.dequant_rows(p.codes, sabs, zabs, rows).T
        cols = rows if p.row_perm is None else np.asarray(p.row_perm, dtype=np.int64)[rows]
        got = Y[np.ix_(mr, cols)].astype(np.float64)
        err = np.abs(got - ref)
        T = V64 @ sabs[half_group][:, rows].astype(np.float64)
        tol = elementwise_tolerance(M, K, ref, A, B, X1, T)
        ratio = err / tol
        k = int(np.argmax(ratio))
        if ratio.flat[k] > worst[0]:
            worst = (float(ratio.flat[k]), (int(mr[k // rows.size]), int(rows[k % rows.size]), float(got.flat[k]),
                                            float(ref.flat[k]), float(tol.flat[k])))
        assert not elementwise or worst[0] <= 1.0, f"element (m, reordered feature, got, ref, tol) = {worst[1]} exceeds its bound"
        num += float((err ** 2).sum())
        den += float((ref ** 2).sum())
        if whole_tile_rows:
            assert rows.size % 128 == 0 and rows[0] % 128 == 0
            e2 = (err ** 2).reshape(mr.size, -1, 128).sum(axis=(0, 2))
            r2 = (ref ** 2).reshape(mr.size, -1, 128).sum(axis=(0, 2))
            bad = np.nonzero(e2 > (TOL ** 2) * r2)[0]
            assert bad.size == 0, f"tile rows {(rows[0] // 128 + bad).tolist()} exceed {TOL} on their own"
    rel = float(np.sqrt(num / den)) if den > 0 else float(np.sqrt(num))
    assert rel <= TOL, rel
    return rel
