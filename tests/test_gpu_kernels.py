"""Per-kernel parity: every HIP kernel, called through the C ABI, against the CPU oracle.

Inputs are seeded draws rounded to the storage type first, so both sides see the same
values; the oracle works in fp64.  Tolerances: 2e-2 relative (bf16 storage), 1e-4 (fp32),
as relative L2 error per tensor plus a max-abs bound of 10 * tol * RMS(oracle).
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from oracle import templora_oracle as O  # noqa: E402
from paper_2401_11504_amd import synth  # noqa: E402

BF16_TOL, F32_TOL = 2e-2, 1e-4


@pytest.fixture(scope="module")
def api():
    from paper_2401_11504_amd import api as _api
    return _api


@pytest.fixture(scope="module")
def H():
    from paper_2401_11504_amd import harness
    return harness


def check(gpu, ref, tol, name="", zero_atol=0.0, per_row=False):
    """per_row: the max-abs criterion is applied row by row, each row (token) against 10 * tol * its own RMS, instead of
    against the RMS of the whole tensor.  For tensors whose rows differ in scale by orders of magnitude (dK and dV of a
    5120-token causal attention: the first key is seen by 5120 queries, the last by one; row RMS 0.7 against 3e-4) the
    whole-tensor RMS is set by the many small rows and 10 * tol * RMS falls below two bf16 roundings of the large
    entries, which no bf16 output can meet; per row the criterion keeps its meaning on large and small rows alike.
    zero_atol: what |gpu| may reach where the oracle is identically zero.  0 (the default) for zeros that follow from
    a zero operand (B = 0 gives dH = s dY 0, hence dA = 0 in any arithmetic); a caller passes a small absolute bound
    only where the oracle's zero is a cancellation x - x that fp32 sums taken in two orders reproduce to rounding."""
    gpu, ref = np.asarray(gpu, np.float64), np.asarray(ref, np.float64)
    assert gpu.shape == ref.shape, (name, gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), name
    nr = np.linalg.norm(ref)
    if nr == 0:
        assert np.all(np.abs(gpu) <= zero_atol), name
        return
    rel = np.linalg.norm(gpu - ref) / nr
    rms = nr / np.sqrt(ref.size)
    mx = np.abs(gpu - ref).max()
    assert rel <= tol, f"{name}: rel L2 {rel:.3e} > {tol}"
    if per_row and ref.ndim == 2:
        row_rms = np.sqrt(np.mean(ref * ref, axis=1))
        row_mx = np.abs(gpu - ref).max(axis=1)
        live = row_rms > 0
        worst = np.max(row_mx[live] / (10 * tol * row_rms[live]))
        assert worst <= 1.0, f"{name}: a row's max abs error is {worst:.3f} x (10 tol x that row's RMS)"
        # a row that is identically zero in the oracle (dq of position 0: one key, dS = x - x) is a cancellation in
        # fp32: rounding noise relative to the tensor's scale
        assert np.all(np.abs(gpu[~live]) <= 1e-5 * np.abs(ref).max()), name
        return
    assert mx <= 10 * tol * rms, f"{name}: max abs {mx:.3e} > {10 * tol * rms:.3e}"


def rnd(seed, shape, std=1.0, bf16=True):
    return synth.normal(seed, (77, len(shape), shape[0]), shape, std, bf16)


# ------------------------------------------------------------------ GEMM NT
@pytest.mark.parametrize("M,N,K,K2", [(128, 128, 64, 0), (1024, 512, 256, 16), (300, 200, 136, 8),
                                      (77, 16, 264, 0), (1024, 64, 1024, 0), (256, 4096, 512, 64), (1, 8, 8, 0)])
def test_gemm_nt_bf16(api, H, M, N, K, K2):
    A, B = rnd(1, (M, K)), rnd(2, (N, K), 0.05)
    A2 = rnd(3, (M, K2)) if K2 else None
    B2 = rnd(4, (N, K2), 0.05) if K2 else None
    ref = A.astype(np.float64) @ B.T.astype(np.float64)
    if K2:
        ref = ref + A2.astype(np.float64) @ B2.T.astype(np.float64)
    Cd = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    api.tl_k_gemm_nt(H.to_dev_bf16(A), H.to_dev_bf16(B), Cd, H.to_dev_bf16(A2) if K2 else None,
                     H.to_dev_bf16(B2) if K2 else None, alpha=0.5)
    torch.cuda.synchronize()
    check(H.bf16_to_np(Cd), 0.5 * ref, BF16_TOL, "C bf16")
    # fp32 output with residual
    R = rnd(5, (M, N), 1.0, False)
    Cf = torch.empty(M, N, dtype=torch.float32, device="cuda")
    api.tl_k_gemm_nt(H.to_dev_bf16(A), H.to_dev_bf16(B), Cf, H.to_dev_bf16(A2) if K2 else None,
                     H.to_dev_bf16(B2) if K2 else None, alpha=1.0, R=H.to_dev_f32(R))
    torch.cuda.synchronize()
    check(Cf.cpu().numpy(), ref + R, 1e-3, "C f32 + R")   # bf16 products are exact; only fp32 summation order differs


@pytest.mark.parametrize("M,N,K", [(1024, 64, 4096), (1000, 192, 1024), (333, 72, 512), (16, 8, 2048), (1024, 128, 11008)])
def test_gemm_nt_skinny(api, H, M, N, K):
    """Small-N, long-K products (the shape of the LoRA down-projections)."""
    A, B = rnd(1, (M, K)), rnd(2, (N, K), 0.05)
    ref = A.astype(np.float64) @ B.T.astype(np.float64)
    Cd = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    api.tl_k_gemm_nt(H.to_dev_bf16(A), H.to_dev_bf16(B), Cd, alpha=0.25)
    R = rnd(5, (M, N), 1.0, False)
    Cf = torch.empty(M, N, dtype=torch.float32, device="cuda")
    api.tl_k_gemm_nt(H.to_dev_bf16(A), H.to_dev_bf16(B), Cf, alpha=1.0, R=H.to_dev_f32(R))
    torch.cuda.synchronize()
    check(H.bf16_to_np(Cd), 0.25 * ref, BF16_TOL, "C bf16")
    check(Cf.cpu().numpy(), ref + R, 1e-3, "C f32 + R")


# One shape (ragged where the instance allows it) for every tile configuration the launcher can pick, with and without
# scratch for a split contraction; `plan` is what tl_k_gemm_nt_plan must report for it, so that a change of the
# selection rules cannot silently leave an instance untested.  K >= 512 runs the interleaved steady-state loop of the
# direct-to-LDS instances, K = 128 their short-contraction fallback.
NT_CASES = [
    # M, N, K, K2, workspace, plan
    (1024, 2048, 512, 64, False, ("128x128", 1)),
    (1000, 2056, 128, 0, False, ("128x128", 1)),
    (520, 4104, 576, 128, False, ("128x128", 1)),
    (2048, 4096, 512, 64, False, ("256x128", 1)),
    (1000, 8184, 128, 64, False, ("256x128", 1)),
    (1000, 4072, 11008, 64, True, ("256x128-split", 2)),
    (1000, 11008, 576, 64, False, ("256x192", 1)),
    (1024, 12288, 128, 0, False, ("256x192", 1)),
    (1000, 16200, 512, 64, False, ("256x256", 1)),
    (1024, 16384, 64, 64, False, ("256x256", 1)),
    (1000, 4104, 72, 8, False, ("reg-128x128", 1)),
    (1024, 1600, 72, 0, False, ("reg-128x64", 1)),
    (1000, 192, 1024, 0, True, ("64x64-split", 4)),
    (1000, 192, 1024, 0, False, ("64x64", 1)),
    (1000, 72, 1032, 0, True, ("reg-64x64-split", 4)),
    (300, 200, 136, 8, False, ("reg-64x64", 1)),
]


def test_gemm_nt_cases_cover_every_configuration(api):
    names = {api.tl_k_gemm_nt_plan(M, N, K, K2, (1 << 26) if ws else 0)[0] for M, N, K, K2, ws, _ in NT_CASES}
    assert names == {"128x128", "256x128", "256x128-split", "256x192", "256x256", "reg-128x128", "reg-128x64", "64x64",
                     "64x64-split", "reg-64x64", "reg-64x64-split"}


@pytest.mark.parametrize("M,N,K,K2,ws,plan", NT_CASES)
def test_gemm_nt_every_configuration(api, H, M, N, K, K2, ws, plan):
    """Each tile configuration of the frozen-weight GEMM on a shape the launcher sends to it."""
    assert api.tl_k_gemm_nt_plan(M, N, K, K2, (1 << 26) if ws else 0)[:2] == plan
    A, B = rnd(1, (M, K)), rnd(2, (N, K), 0.05)
    A2 = rnd(3, (M, K2)) if K2 else None
    B2 = rnd(4, (N, K2), 0.05) if K2 else None
    ref = A.astype(np.float64) @ B.T.astype(np.float64)
    if K2:
        ref = ref + A2.astype(np.float64) @ B2.T.astype(np.float64)
    R = rnd(5, (M, N), 1.0, False)
    scratch = torch.empty(1 << 26, dtype=torch.float32, device="cuda") if ws else None
    Cf = torch.empty(M, N, dtype=torch.float32, device="cuda")
    api.tl_k_gemm_nt(H.to_dev_bf16(A), H.to_dev_bf16(B), Cf, H.to_dev_bf16(A2) if K2 else None,
                     H.to_dev_bf16(B2) if K2 else None, alpha=1.0, R=H.to_dev_f32(R), workspace=scratch)
    Cb = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    api.tl_k_gemm_nt(H.to_dev_bf16(A), H.to_dev_bf16(B), Cb, H.to_dev_bf16(A2) if K2 else None,
                     H.to_dev_bf16(B2) if K2 else None, alpha=0.5, workspace=scratch)
    torch.cuda.synchronize()
    check(Cf.cpu().numpy(), ref + R, 1e-3, "C f32 + R")   # bf16 products are exact; only fp32 summation order differs
    check(H.bf16_to_np(Cb), 0.5 * ref, BF16_TOL, "C bf16")


def test_gemm_nt_two_column_ranges(api, H):
    """The gate|up shape at 1024 tokens: the launcher sends it out as two launches over two column ranges (whole rounds
    of 256x256 tiles, then the rest).  Checked on sampled columns, among them those on both sides of the seam."""
    M, N, K, K2 = 1024, 22016, 4096, 128
    A, B = rnd(1, (M, K)), rnd(2, (N, K), 0.05)
    A2, B2 = rnd(3, (M, K2)), rnd(4, (N, K2), 0.05)
    rs = np.random.default_rng(7)
    cols = np.unique(np.concatenate([rs.choice(N, 384, replace=False), np.arange(16384 - 40, 16384 + 40),
                                     np.arange(8192 - 8, 8192 + 8), [0, N - 1]]))
    ref = A.astype(np.float64) @ B[cols].T.astype(np.float64) + A2.astype(np.float64) @ B2[cols].T.astype(np.float64)
    Cd = torch.zeros(M, N, dtype=torch.bfloat16, device="cuda")
    api.tl_k_gemm_nt(H.to_dev_bf16(A), H.to_dev_bf16(B), Cd, H.to_dev_bf16(A2), H.to_dev_bf16(B2))
    torch.cuda.synchronize()
    check(H.bf16_to_np(Cd)[:, cols], ref, BF16_TOL, "C bf16")
    R = rnd(5, (M, N), 1.0, False)
    Cf = torch.zeros(M, N, dtype=torch.float32, device="cuda")
    api.tl_k_gemm_nt(H.to_dev_bf16(A), H.to_dev_bf16(B), Cf, H.to_dev_bf16(A2), H.to_dev_bf16(B2), alpha=1.0, R=H.to_dev_f32(R))
    torch.cuda.synchronize()
    check(Cf.cpu().numpy()[:, cols], ref + R[:, cols], 1e-3, "C f32 + R")


def test_gemm_nt_strided_operands(api, H):
    # operands that are column blocks of wider buffers (as q|k|v and gate|up are)
    M, N, K = 200, 96, 128
    Aw, Bw = rnd(1, (M, 3 * K)), rnd(2, (N, 2 * K), 0.05)
    Ad, Bd = H.to_dev_bf16(Aw), H.to_dev_bf16(Bw)
    Cw = torch.zeros(M, 2 * N, dtype=torch.bfloat16, device="cuda")
    api.tl_k_gemm_nt(Ad[:, K:2 * K], Bd[:, K:], Cw[:, N:])
    torch.cuda.synchronize()
    ref = Aw[:, K:2 * K].astype(np.float64) @ Bw[:, K:].T.astype(np.float64)
    check(H.bf16_to_np(Cw[:, N:]), ref, BF16_TOL)
    assert torch.all(Cw[:, :N] == 0)


# ------------------------------------------------------------------ GEMM TN
@pytest.mark.parametrize("T,Mo,No", [(64, 64, 64), (1024, 48, 256), (300, 200, 136), (1000, 16, 704), (5, 8, 8)])
def test_gemm_tn(api, H, T, Mo, No):
    P, Q = rnd(1, (T, Mo)), rnd(2, (T, No))
    C = torch.empty(Mo, No, dtype=torch.float32, device="cuda")
    api.tl_k_gemm_tn(H.to_dev_bf16(P), H.to_dev_bf16(Q), C, alpha=2.0)
    torch.cuda.synchronize()
    check(C.cpu().numpy(), 2.0 * P.T.astype(np.float64) @ Q.astype(np.float64), 1e-3)


# ------------------------------------------------------------------ RMSNorm
@pytest.mark.parametrize("T,d", [(5, 64), (130, 1024), (33, 4096), (7, 8192), (3, 12288)])
def test_rmsnorm_fwd_bwd(api, H, T, d):
    h = rnd(1, (T, d), 2.0, False)
    g = 1.0 + 0.1 * rnd(2, (d,), 1.0, False)
    dy = rnd(3, (T, d))
    dres = rnd(4, (T, d), 1.0, False)
    y = torch.empty(T, d, dtype=torch.bfloat16, device="cuda")
    api.tl_k_rmsnorm_fwd(H.to_dev_f32(h), H.to_dev_f32(g), 1e-5, y)
    dh = torch.empty(T, d, dtype=torch.float32, device="cuda")
    dhb = torch.empty(T, d, dtype=torch.bfloat16, device="cuda")
    api.tl_k_rmsnorm_bwd(H.to_dev_bf16(dy), H.to_dev_f32(h), H.to_dev_f32(g), H.to_dev_f32(dres), 1e-5, dh, dhb)
    torch.cuda.synchronize()
    check(H.bf16_to_np(y), O.rmsnorm_fwd(h, g, 1e-5), BF16_TOL, "y")
    ref = dres + O.rmsnorm_bwd(dy, h, g, 1e-5)
    check(dh.cpu().numpy(), ref, F32_TOL, "dh")
    check(H.bf16_to_np(dhb), ref, BF16_TOL, "dh bf16")
    dh2 = torch.empty_like(dh)
    api.tl_k_rmsnorm_bwd(H.to_dev_bf16(dy), H.to_dev_f32(h), H.to_dev_f32(g), None, 1e-5, dh2, None)
    torch.cuda.synchronize()
    check(dh2.cpu().numpy(), O.rmsnorm_bwd(dy, h, g, 1e-5), F32_TOL, "dh without residual")


# ------------------------------------------------------------------ RoPE
@pytest.mark.parametrize("T,nh,dh,pos0", [(70, 3, 64, 0), (1024, 2, 128, 0), (9, 1, 64, 1000)])
def test_rope(api, H, T, nh, dh, pos0):
    x = rnd(1, (T, nh * dh))
    xd = H.to_dev_bf16(x)
    api.tl_k_rope(xd, nh, dh, 10000.0, pos0, +1)
    torch.cuda.synchronize()
    ref = O.rope_fwd(x.reshape(T, nh, dh), 10000.0, pos0).reshape(T, nh * dh)
    check(H.bf16_to_np(xd), ref, BF16_TOL, "fwd")
    xb = H.to_dev_bf16(x)
    api.tl_k_rope(xb, nh, dh, 10000.0, pos0, -1)
    torch.cuda.synchronize()
    check(H.bf16_to_np(xb), O.rope_bwd(x.reshape(T, nh, dh), 10000.0, pos0).reshape(T, nh * dh), BF16_TOL, "bwd")


@pytest.mark.parametrize("T,nh,dh,pos0,ld_extra", [(70, 3, 64, 0, 0), (1024, 2, 128, 0, 0), (9, 1, 64, 1000, 0),
                                                   (130, 2, 128, 7, 256),      # a slice of a wider buffer (q | k of q|k|v)
                                                   (33, 2, 24, 0, 0)])         # head width no multiple of 16: scalar kernel
def test_rope_through_the_angle_table(api, H, T, nh, dh, pos0, ld_extra):
    """The chunk path rotates q and k with a (cos, sin) table built in fp64 and 16-byte accesses; same bar as above."""
    x = rnd(2, (T, nh * dh + ld_extra))
    table = torch.empty((pos0 + T) * dh, dtype=torch.float32, device="cuda")
    for sign, ref_fn in ((+1, O.rope_fwd), (-1, O.rope_bwd)):
        xd = H.to_dev_bf16(x)
        api.tl_k_rope_table(xd[:, :nh * dh], nh, dh, table, 10000.0, pos0, sign)
        torch.cuda.synchronize()
        got = H.bf16_to_np(xd)
        ref = ref_fn(x[:, :nh * dh].reshape(T, nh, dh), 10000.0, pos0).reshape(T, nh * dh)
        check(got[:, :nh * dh], ref, BF16_TOL, f"sign {sign}")
        assert np.array_equal(got[:, nh * dh:], H.bf16_to_np(H.to_dev_bf16(x))[:, nh * dh:])   # columns beyond the heads untouched
    with pytest.raises(api.TlError):
        api.tl_k_rope_table(H.to_dev_bf16(x)[:, :nh * dh], nh, dh, table[:8], 10000.0, pos0, +1)


# ------------------------------------------------------------------ SwiGLU
@pytest.mark.parametrize("T,f", [(3, 8), (257, 704), (64, 11008)])
def test_swiglu(api, H, T, f):
    gu, da = rnd(1, (T, 2 * f), 2.0), rnd(2, (T, f))
    a = torch.empty(T, f, dtype=torch.bfloat16, device="cuda")
    dgu = torch.empty(T, 2 * f, dtype=torch.bfloat16, device="cuda")
    api.tl_k_swiglu_fwd(H.to_dev_bf16(gu), a)
    api.tl_k_swiglu_bwd(H.to_dev_bf16(da), H.to_dev_bf16(gu), dgu)
    torch.cuda.synchronize()
    check(H.bf16_to_np(a), O.swiglu_fwd(gu[:, :f], gu[:, f:]), BF16_TOL, "a")
    dg, du = O.swiglu_bwd(da, gu[:, :f], gu[:, f:])
    check(H.bf16_to_np(dgu), np.concatenate([dg, du], 1), BF16_TOL, "dgu")


# ------------------------------------------------------------------ attention
# the last case has more workgroups than the chip has CUs (9 query blocks x 30 heads, ragged): the forward kernel then
# hands its blocks out heaviest first, a different block-to-workgroup mapping from the one-round cases
# (4096 and 5120 tokens: the longest training samples of the paper's Table 5, Delta = 4096 behind L_T = 1024)
@pytest.mark.parametrize("T,nh,dh", [(64, 1, 64), (200, 2, 64), (333, 2, 128), (1024, 2, 128), (1, 1, 64), (129, 1, 128),
                                     (1100, 30, 64), (4096, 2, 128), (5120, 2, 128), (5120, 1, 64)])
def test_attention_fwd_bwd(api, H, T, nh, dh):
    qkv = rnd(1, (T, 3 * nh * dh), 1.0)
    do = rnd(2, (T, nh * dh))
    d = nh * dh
    qkvd = H.to_dev_bf16(qkv)
    o = torch.zeros(T, d, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(nh, T, dtype=torch.float32, device="cuda")
    api.tl_k_attention_fwd(qkvd[:, :d], qkvd[:, d:2 * d], qkvd[:, 2 * d:], nh, dh, o, lse)
    torch.cuda.synchronize()
    q, k, v = (qkv[:, i * d:(i + 1) * d].reshape(T, nh, dh) for i in range(3))
    ro, P = O.attention_fwd(q, k, v)
    check(H.bf16_to_np(o), ro.reshape(T, d), BF16_TOL, "o")
    S = np.einsum("thd,uhd->htu", q.astype(np.float64), k.astype(np.float64)) / np.sqrt(dh)
    S = np.where(np.triu(np.ones((T, T), bool), 1)[None], -np.inf, S)
    mx = S.max(-1)
    ref_lse = np.log(np.exp(S - mx[..., None]).sum(-1)) + mx
    assert np.abs(lse.cpu().numpy() - ref_lse).max() < 2e-3
    # backward takes the GPU's own (bf16-rounded) o, as the composed path does
    dqkv = torch.zeros(T, 3 * d, dtype=torch.bfloat16, device="cuda")
    delta = torch.zeros(nh, T, dtype=torch.float32, device="cuda")
    api.tl_k_attention_bwd(qkvd[:, :d], qkvd[:, d:2 * d], qkvd[:, 2 * d:], o, H.to_dev_bf16(do), lse, nh, dh,
                           dqkv[:, :d], dqkv[:, d:2 * d], dqkv[:, 2 * d:], delta)
    torch.cuda.synchronize()
    dq, dk, dv = O.attention_bwd(do.reshape(T, nh, dh), q, k, v, P)
    g = H.bf16_to_np(dqkv)
    check(g[:, :d], dq.reshape(T, d), BF16_TOL, "dq", per_row=True)
    check(g[:, d:2 * d], dk.reshape(T, d), BF16_TOL, "dk", per_row=True)
    check(g[:, 2 * d:], dv.reshape(T, d), BF16_TOL, "dv", per_row=True)


# ------------------------------------------------------------------ cross entropy
@pytest.mark.parametrize("T,V,n_ctx", [(9, 64, 0), (130, 1000, 0), (64, 32000, 0), (40, 776, 17)])
def test_cross_entropy(api, H, T, V, n_ctx):
    z = rnd(1, (T, V), 1.5, False)
    tok = synth.uniform_tokens(3, T, V)
    labels, mask, N = O.labels_and_mask(tok, n_ctx)
    first = max(n_ctx, 1) - 1
    assert np.array_equal(np.nonzero(mask)[0], np.arange(first, T - 1))
    nll = torch.zeros(T, dtype=torch.float32, device="cuda")
    dl = torch.zeros(T, V, dtype=torch.bfloat16, device="cuda")
    ls = torch.zeros(4, dtype=torch.float32, device="cuda")
    lab_d = torch.from_numpy(labels.astype(np.int32)).cuda()
    api.tl_k_cross_entropy(H.to_dev_f32(z), lab_d, first, N, nll, dl, ls)
    torch.cuda.synchronize()
    loss, rnll, rdl = O.cross_entropy(z, labels, mask)
    check(nll.cpu().numpy(), rnll, F32_TOL, "nll")
    assert abs(ls[0].item() / N - loss) <= F32_TOL * loss
    check(H.bf16_to_np(dl), rdl, BF16_TOL, "dlogits")
    assert torch.all(dl[~torch.from_numpy(mask).cuda()] == 0)


# ------------------------------------------------------------------ AdamW
@pytest.mark.parametrize("n", [7, 4096, 1_000_003])
def test_adamw_steps(api, H, n):
    p = rnd(1, (n,), 0.02, False)
    m, v = np.zeros(n), np.zeros(n)
    pd, md, vd = H.to_dev_f32(p), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    sh = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    pr = p.astype(np.float64)
    for step in (1, 2, 3):
        g = rnd(10 + step, (n,), 1e-3, False)
        g[::5] = 0.0
        api.tl_k_adamw(pd, H.to_dev_f32(g), md, vd, sh, step, 5e-5, 0.9, 0.999, 1e-8, 0.01)
        pr, m, v = O.adamw_step(pr, g, m, v, step, 5e-5, 0.9, 0.999, 1e-8, 0.01)
    torch.cuda.synchronize()
    check(pd.cpu().numpy() - p, pr - p, 1e-3, "delta p")      # the update itself, not p, carries the comparison
    check(md.cpu().numpy(), m, F32_TOL, "m")
    check(vd.cpu().numpy(), v, F32_TOL, "v")
    assert torch.equal(sh, pd.bfloat16())


def test_adamw_zero_grad_leaves_param_bit_identical(api, H):
    p = rnd(1, (1000,), 0.02, False)
    pd = H.to_dev_f32(p)
    api.tl_k_adamw(pd, torch.zeros(1000, device="cuda"), torch.zeros(1000, device="cuda"),
                   torch.zeros(1000, device="cuda"), None, 1, 5e-5)
    torch.cuda.synchronize()
    assert np.array_equal(pd.cpu().numpy(), p)


# ------------------------------------------------------------------ embedding gather (bit exact)
def test_embed_rows_bit_exact(api, H):
    V, d, T = 1000, 256, 77
    E = rnd(1, (V, d), 0.02)
    tok = synth.uniform_tokens(5, T, V)
    h = torch.zeros(T, d, device="cuda")
    api.tl_k_embed(H.to_dev_bf16(E), torch.from_numpy(tok).cuda(), h)
    torch.cuda.synchronize()
    assert np.array_equal(h.cpu().numpy(), E[tok])
