"""Op-level GPU parity through the C ABI: each kernel against the definition evaluated in
float64 on the same (already rounded) inputs.  These also run at the full benchmark shapes,
where the oracle cannot run end to end: there, sampled output entries are checked one by one.
"""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import stage_oracle as so
from paper_2412_14374_amd import binding as B
from paper_2412_14374_amd import inputs as inp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def rel_l2(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV).to(dtype).contiguous()


def host(t):
    return t.detach().to(torch.float64).cpu().numpy()


def stream():
    return torch.cuda.current_stream().cuda_stream


GEMM_SHAPES = [
    # M, N, K  (multiples of 8; tails against the 256/128 tiles and the 64-wide k step)
    (8, 8, 8), (136, 72, 200), (256, 256, 64), (264, 520, 328), (512, 384, 1000), (1032, 776, 72),
]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("aks,bks", [(0, 0), (0, 1), (1, 1), (1, 0)])
def test_gemm_bf16_all_layouts_and_epilogues(M, N, K, aks, bks):
    rng = np.random.default_rng(M * 7 + N * 3 + K + aks * 2 + bks)
    A = inp.round_to_dtype(rng.standard_normal((M, K)), inp.DT_BF16)
    Bm = inp.round_to_dtype(rng.standard_normal((N, K)), inp.DT_BF16)
    bias = inp.round_to_dtype(rng.standard_normal(N), inp.DT_BF16)
    res = inp.round_to_dtype(rng.standard_normal((M, N)), inp.DT_BF16)
    ref = A @ Bm.T
    At = dev(A.T if aks else A, torch.bfloat16)
    Bt = dev(Bm.T if bks else Bm, torch.bfloat16)
    lda = M if aks else K
    ldb = N if bks else K
    bt, rt = dev(bias, torch.bfloat16), dev(res, torch.bfloat16)
    # store bf16 with bias + residual
    Cb = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
    B.jpp_op_gemm(B.JPP_BF16, M, N, K, At.data_ptr(), lda, aks, Bt.data_ptr(), ldb, bks, Cb.data_ptr(), N,
                  B.OUT_STORE, bt.data_ptr(), rt.data_ptr(), stream())
    # store fp32, no epilogue terms
    Cf = torch.full((M, N), 7.0, dtype=torch.float32, device=DEV)
    B.jpp_op_gemm(B.JPP_BF16, M, N, K, At.data_ptr(), lda, aks, Bt.data_ptr(), ldb, bks, Cf.data_ptr(), N,
                  B.OUT_STORE_F32, None, None, stream())
    # accumulate into fp32 twice
    Ca = torch.ones((M, N), dtype=torch.float32, device=DEV)
    for _ in range(2):
        B.jpp_op_gemm(B.JPP_BF16, M, N, K, At.data_ptr(), lda, aks, Bt.data_ptr(), ldb, bks, Ca.data_ptr(), N,
                      B.OUT_ACC_F32, None, None, stream())
    torch.cuda.synchronize()
    assert rel_l2(host(Cf), ref) < 1e-5                       # fp32 accumulate of exact bf16 products
    assert np.abs(host(Cf) - ref).max() < 1e-3 * math.sqrt(K)
    assert rel_l2(host(Ca), 1.0 + 2 * ref) < 1e-5
    assert rel_l2(host(Cb), ref + bias[None, :] + res) < 4e-3  # one bf16 rounding of the result


@pytest.mark.parametrize("variant", [1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("aks,bks", [(0, 0), (0, 1), (1, 1), (1, 0)])
def test_gemm_bf16_every_tile_configuration_gives_the_same_bits(variant, aks, bks):
    """The automatic choice depends on the shape, so each configuration is forced in turn on
    shapes with ragged tails in every dimension: all three output modes must match the
    definition and agree bit for bit with the automatic choice (same k order per element)."""
    rng = np.random.default_rng(100 + aks * 2 + bks)
    for (M, N, K) in [(264, 520, 328), (776, 136, 72)]:
        A = inp.round_to_dtype(rng.standard_normal((M, K)), inp.DT_BF16)
        Bm = inp.round_to_dtype(rng.standard_normal((N, K)), inp.DT_BF16)
        bias = inp.round_to_dtype(rng.standard_normal(N), inp.DT_BF16)
        res = inp.round_to_dtype(rng.standard_normal((M, N)), inp.DT_BF16)
        At = dev(A.T if aks else A, torch.bfloat16)
        Bt = dev(Bm.T if bks else Bm, torch.bfloat16)
        bt, rt = dev(bias, torch.bfloat16), dev(res, torch.bfloat16)
        lda, ldb = (M if aks else K), (N if bks else K)
        out = {}
        try:
            for v in (0, variant):
                B.jpp_set_gemm_variant(v)
                Cb = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
                Cf = torch.full((M, N), 7.0, dtype=torch.float32, device=DEV)
                Ca = torch.ones((M, N), dtype=torch.float32, device=DEV)
                a = (B.JPP_BF16, M, N, K, At.data_ptr(), lda, aks, Bt.data_ptr(), ldb, bks)
                B.jpp_op_gemm(*a, Cb.data_ptr(), N, B.OUT_STORE, bt.data_ptr(), rt.data_ptr(), stream())
                B.jpp_op_gemm(*a, Cf.data_ptr(), N, B.OUT_STORE_F32, None, None, stream())
                B.jpp_op_gemm(*a, Ca.data_ptr(), N, B.OUT_ACC_F32, None, None, stream())
                torch.cuda.synchronize()
                out[v] = (Cb, Cf, Ca)
        finally:
            B.jpp_set_gemm_variant(0)
        ref = A @ Bm.T
        assert rel_l2(host(out[variant][1]), ref) < 1e-5
        assert rel_l2(host(out[variant][2]), 1.0 + ref) < 1e-5
        assert rel_l2(host(out[variant][0]), ref + bias[None, :] + res) < 4e-3
        for got, auto in zip(out[variant], out[0]):
            assert torch.equal(got, auto)


SPLIT_SHAPES = [
    # M, N, K: few output tiles and a long k, so that the launch is split along k
    (264, 520, 1000), (512, 384, 1000), (1032, 776, 2056), (8, 8, 4096), (136, 72, 520),
]


@pytest.mark.parametrize("M,N,K", SPLIT_SHAPES)
@pytest.mark.parametrize("aks,bks", [(0, 0), (0, 1), (1, 1), (1, 0)])
def test_gemm_bf16_split_along_k_with_scratch(M, N, K, aks, bks):
    """jpp_op_gemm_ws: partial tiles through the scratch buffer, summed by the second kernel
    with bias, residual and rounding.  Checked against the definition; the scratch is sized by
    jpp_op_gemm_workspace_bytes, and a too small one must fall back to the unsplit launch."""
    rng = np.random.default_rng(M + 3 * N + K + aks * 2 + bks)
    A = inp.round_to_dtype(rng.standard_normal((M, K)), inp.DT_BF16)
    Bm = inp.round_to_dtype(rng.standard_normal((N, K)), inp.DT_BF16)
    bias = inp.round_to_dtype(rng.standard_normal(N), inp.DT_BF16)
    res = inp.round_to_dtype(rng.standard_normal((M, N)), inp.DT_BF16)
    ref = A @ Bm.T
    At = dev(A.T if aks else A, torch.bfloat16)
    Bt = dev(Bm.T if bks else Bm, torch.bfloat16)
    lda, ldb = (M if aks else K), (N if bks else K)
    bt, rt = dev(bias, torch.bfloat16), dev(res, torch.bfloat16)
    need = B.jpp_op_gemm_workspace_bytes(B.JPP_BF16, M, N, K, B.OUT_STORE)
    assert need > 0                                           # these shapes are meant to split
    need_acc = B.jpp_op_gemm_workspace_bytes(B.JPP_BF16, M, N, K, B.OUT_ACC_F32)
    # accumulating outputs are cut when that fills at least a twentieth more of the chip with
    # ranges of 16 k-steps or more: of these shapes only 63 tiles of 128 x 128 with 33 k-steps
    assert (need_acc > 0) == ((M, N, K) == (1032, 776, 2056))
    ws = torch.full((need // 4 + 64,), float("nan"), dtype=torch.float32, device=DEV)
    a = (B.JPP_BF16, M, N, K, At.data_ptr(), lda, aks, Bt.data_ptr(), ldb, bks)
    Cb = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
    Cf = torch.full((M, N), 7.0, dtype=torch.float32, device=DEV)
    Cs = torch.full((M, N), 7.0, dtype=torch.float32, device=DEV)
    Cu = torch.full((M, N), 7.0, dtype=torch.float32, device=DEV)
    B.jpp_op_gemm_ws(*a, Cb.data_ptr(), N, B.OUT_STORE, bt.data_ptr(), rt.data_ptr(), ws.data_ptr(), need, stream())
    B.jpp_op_gemm_ws(*a, Cf.data_ptr(), N, B.OUT_STORE_F32, None, None, ws.data_ptr(), need, stream())
    B.jpp_op_gemm_ws(*a, Cs.data_ptr(), N, B.OUT_STORE_F32, None, None, ws.data_ptr(), need - 16, stream())
    B.jpp_op_gemm(*a, Cu.data_ptr(), N, B.OUT_STORE_F32, None, None, stream())
    torch.cuda.synchronize()
    assert rel_l2(host(Cf), ref) < 1e-5
    assert np.abs(host(Cf) - ref).max() < 1e-3 * math.sqrt(K)
    assert rel_l2(host(Cb), ref + bias[None, :] + res) < 4e-3
    assert torch.equal(Cs, Cu)                                # scratch too small: the unsplit launch
    assert bool(torch.isnan(ws[need // 4:]).all())            # nothing written past the stated size
    if need_acc:
        # the accumulating mode cut along k: the partial sums are added to C once per launch
        wa = torch.full((need_acc // 4 + 64,), float("nan"), dtype=torch.float32, device=DEV)
        Ca = torch.ones((M, N), dtype=torch.float32, device=DEV)
        Cv = torch.ones((M, N), dtype=torch.float32, device=DEV)
        Cw = torch.ones((M, N), dtype=torch.float32, device=DEV)
        for _ in range(2):
            B.jpp_op_gemm_ws(*a, Ca.data_ptr(), N, B.OUT_ACC_F32, None, None, wa.data_ptr(), need_acc, stream())
        B.jpp_op_gemm_ws(*a, Cv.data_ptr(), N, B.OUT_ACC_F32, None, None, wa.data_ptr(), need_acc - 16, stream())
        B.jpp_op_gemm(*a, Cw.data_ptr(), N, B.OUT_ACC_F32, None, None, stream())
        torch.cuda.synchronize()
        assert rel_l2(host(Ca), 1.0 + 2 * ref) < 1e-5
        assert np.abs(host(Ca) - (1.0 + 2 * ref)).max() < 2e-3 * math.sqrt(K)
        assert torch.equal(Cv, Cw)
        assert bool(torch.isnan(wa[need_acc // 4:]).all())


SPLIT_FULL = [
    # benchmark-size GEMMs whose last round of 256 x 256 tiles is half empty
    ("ffn-down fwd", 2048, 12288, 49152, 0, 0), ("ffn-up dgrad", 2048, 12288, 49152, 0, 1),
    ("qkv fwd", 2048, 36864, 12288, 0, 0), ("attn-out fwd", 2048, 12288, 12288, 0, 0),
]


@pytest.mark.parametrize("name,M,N,K,aks,bks", SPLIT_FULL)
def test_gemm_split_full_shape_sampled_entries(name, M, N, K, aks, bks):
    g = torch.Generator(device=DEV)
    g.manual_seed(M + N + K + 1)
    A = torch.randn((K, M) if aks else (M, K), generator=g, device=DEV).to(torch.bfloat16)
    Bm = (torch.randn((K, N) if bks else (N, K), generator=g, device=DEV) * 0.02).to(torch.bfloat16)
    bias = torch.randn(N, generator=g, device=DEV).to(torch.bfloat16)
    res = torch.randn((M, N), generator=g, device=DEV).to(torch.bfloat16)
    need = B.jpp_op_gemm_workspace_bytes(B.JPP_BF16, M, N, K, B.OUT_STORE)
    assert need > 0
    ws = torch.empty(need // 4, dtype=torch.float32, device=DEV)
    Cc = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    B.jpp_op_gemm_ws(B.JPP_BF16, M, N, K, A.data_ptr(), M if aks else K, aks, Bm.data_ptr(), N if bks else K, bks,
                     Cc.data_ptr(), N, B.OUT_STORE, bias.data_ptr(), res.data_ptr(), ws.data_ptr(), need, stream())
    torch.cuda.synchronize()
    rng = np.random.default_rng(1)
    ms = np.concatenate([rng.integers(0, M, 4096), [0, 0, M - 1, M - 1, 255, 256, M - 256, M - 257]])
    ns = np.concatenate([rng.integers(0, N, 4096), [0, N - 1, 0, N - 1, 255, 256, N - 256, N - 257]])
    mi, ni = torch.from_numpy(ms).to(DEV), torch.from_numpy(ns).to(DEV)
    a_rows = (A[:, mi].T if aks else A[mi, :]).float().cpu().numpy().astype(np.float64)
    b_rows = (Bm[:, ni].T if bks else Bm[ni, :]).float().cpu().numpy().astype(np.float64)
    ref = np.einsum("sk,sk->s", a_rows, b_rows) + bias[ni].double().cpu().numpy() + res[mi, ni].double().cpu().numpy()
    got = Cc[mi, ni].double().cpu().numpy()
    assert rel_l2(got, ref) < 4e-3, name
    assert bool(torch.isfinite(Cc.float()).all())


WGRAD_SPLIT_FULL = [
    # weight gradients of the d = 2048 configuration over a group of 8 microbatches: outputs of 192 and
    # 64 tiles of 256 x 256, every tile cut into four ranges of k
    ("qkv wgrad", 6144, 2048, 65536), ("attn-out wgrad", 2048, 2048, 65536),
    # a vocabulary's weight gradient (one microbatch of it): 197 x 16 tiles are 12.3 rounds, the 80 tiles
    # of the last round are cut into three ranges of k, all others accumulate in one pass
    ("head wgrad", 50304, 4096, 4096),
]


@pytest.mark.parametrize("name,M,N,K", WGRAD_SPLIT_FULL)
def test_gemm_wgrad_split_full_shape_sampled_entries(name, M, N, K):
    g = torch.Generator(device=DEV)
    g.manual_seed(M + N + K + 2)
    A = (torch.randn((K, M), generator=g, device=DEV) * 0.01).to(torch.bfloat16)       # cotangents, k-strided
    Bm = torch.randn((K, N), generator=g, device=DEV).to(torch.bfloat16)               # activations, k-strided
    need = B.jpp_op_gemm_workspace_bytes(B.JPP_BF16, M, N, K, B.OUT_ACC_F32)
    tiles = -(-M // 256) * (N // 256)
    assert need == (tiles * 4 if tiles < 512 else (tiles % 256) * 3) * 256 * 256 * 4
    ws = torch.empty(need // 4, dtype=torch.float32, device=DEV)
    G0 = torch.randn((M, N), generator=g, device=DEV)
    outs = []
    for _ in range(2):                                  # twice: the same bits (fixed order, no atomics)
        G = G0.clone()
        B.jpp_op_gemm_ws(B.JPP_BF16, M, N, K, A.data_ptr(), M, 1, Bm.data_ptr(), N, 1, G.data_ptr(), N, B.OUT_ACC_F32,
                         None, None, ws.data_ptr(), need, stream())
        torch.cuda.synchronize()
        outs.append(G)
    assert torch.equal(outs[0], outs[1])
    rng = np.random.default_rng(2)
    # (tiles are numbered along bands of 8 tile rows, so the last tiles of a launch, the ones a
    # tail split cuts, are its last rows: a quarter of the samples come from the last 1024 rows)
    ms = np.concatenate([rng.integers(0, M, 4096), rng.integers(max(0, M - 1024), M, 1024),
                         [0, 0, M - 1, M - 1, 255, 256, M - 256, M - 257]])
    ns = np.concatenate([rng.integers(0, N, 4096 + 1024), [0, N - 1, 0, N - 1, 255, 256, N - 256, N - 257]])
    mi, ni = torch.from_numpy(ms).to(DEV), torch.from_numpy(ns).to(DEV)
    a_cols = A[:, mi].T.float().cpu().numpy().astype(np.float64)
    b_cols = Bm[:, ni].T.float().cpu().numpy().astype(np.float64)
    ref = np.einsum("sk,sk->s", a_cols, b_cols) + G0[mi, ni].double().cpu().numpy()
    got = outs[0][mi, ni].double().cpu().numpy()
    assert rel_l2(got, ref) < 1e-5, name
    assert bool(torch.isfinite(outs[0]).all())


GELU_FUSED_SHAPES = [
    # M, N, K, with workspace (the last round of tiles cut along k, GeLU applied by the fix-up kernel)
    (136, 72, 200, False), (264, 520, 328, False), (1032, 776, 2056, True), (2048, 12288, 2048, True),
]


@pytest.mark.parametrize("M,N,K,with_ws", GELU_FUSED_SHAPES)
@pytest.mark.parametrize("act", [inp.ACT_GELU, inp.ACT_GELU_TANH])
def test_gemm_with_fused_gelu_gives_the_bits_of_the_separate_kernels(M, N, K, with_ws, act):
    """The feed-forward block as the stage runs it: forward, one GEMM writes h = x W1^T + b1 and
    a = gelu(h); backward, one GEMM writes dh = (dy W2) * gelu'(h) without storing dy W2.
    Both against the unfused sequence (jpp_op_gemm, then jpp_op_act_fwd / _bwd): identical
    bits, and against the definition in float64."""
    rng = np.random.default_rng(M + N + K + act)
    x = inp.round_to_dtype(rng.standard_normal((M, K)), inp.DT_BF16)
    w = inp.round_to_dtype(rng.standard_normal((N, K)) * 0.05, inp.DT_BF16)
    b = inp.round_to_dtype(rng.standard_normal(N) * 0.1, inp.DT_BF16)
    xt, wt, bt = dev(x, torch.bfloat16), dev(w, torch.bfloat16), dev(b, torch.bfloat16)
    need = B.jpp_op_gemm_workspace_bytes(B.JPP_BF16, M, N, K, B.OUT_STORE) if with_ws else 0
    assert (need > 0) == with_ws
    ws = torch.empty(max(need // 4, 4), dtype=torch.float32, device=DEV)
    wsp = ws.data_ptr() if need else None
    z = lambda: torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
    h0, a0, h1, a1 = z(), z(), z(), z()
    B.jpp_op_gemm_ws(B.JPP_BF16, M, N, K, xt.data_ptr(), K, 0, wt.data_ptr(), K, 0, h0.data_ptr(), N, B.OUT_STORE,
                     bt.data_ptr(), None, wsp, need, stream())
    B.jpp_op_act_fwd(B.JPP_BF16, act, M, N, h0.data_ptr(), a0.data_ptr(), stream())
    B.jpp_op_gemm_gelu(M, N, K, xt.data_ptr(), K, 0, wt.data_ptr(), K, 0, h1.data_ptr(), N, bt.data_ptr(), act, 0,
                       a1.data_ptr(), wsp, need, stream())
    torch.cuda.synchronize()
    assert torch.equal(h0.view(torch.int16), h1.view(torch.int16))
    assert torch.equal(a0.view(torch.int16), a1.view(torch.int16))
    spec = so.StageSpec(n_layers=1, d_model=8, n_q_heads=1, n_kv_heads=1, head_dim=8, d_ffn=N, seq_len=1,
                        microbatch=1, act=act)
    href = x @ w.T + b[None, :]
    assert rel_l2(host(h1), href) < 4e-3
    assert rel_l2(host(a1), so.act_forward(spec, host(h1))) < 4e-3
    # backward: dy [M, K] times W2 [K, N] (k-strided, as the stage reads it), h from above
    dy = inp.round_to_dtype(rng.standard_normal((M, K)) * 0.01, inp.DT_BF16)
    w2 = inp.round_to_dtype(rng.standard_normal((K, N)) * 0.05, inp.DT_BF16)
    dyt, w2t = dev(dy, torch.bfloat16), dev(w2, torch.bfloat16)
    da0, dh0, dh1 = z(), z(), z()
    B.jpp_op_gemm_ws(B.JPP_BF16, M, N, K, dyt.data_ptr(), K, 0, w2t.data_ptr(), N, 1, da0.data_ptr(), N, B.OUT_STORE,
                     None, None, wsp, need, stream())
    B.jpp_op_act_bwd(B.JPP_BF16, act, M, N, h0.data_ptr(), da0.data_ptr(), dh0.data_ptr(), stream())
    B.jpp_op_gemm_gelu(M, N, K, dyt.data_ptr(), K, 0, w2t.data_ptr(), N, 1, dh1.data_ptr(), N, None, act, 1,
                       h1.data_ptr(), wsp, need, stream())
    torch.cuda.synchronize()
    assert torch.equal(dh0.view(torch.int16), dh1.view(torch.int16))
    assert rel_l2(host(dh1), so.act_backward(spec, host(h1), dy @ w2)) < 6e-3
    with pytest.raises(B.JppError):          # the second tensor must not be the output
        B.jpp_op_gemm_gelu(M, N, K, dyt.data_ptr(), K, 0, w2t.data_ptr(), N, 1, dh1.data_ptr(), N, None, act, 1,
                           dh1.data_ptr(), wsp, need, stream())


def test_gemm_bf16_padded_leading_dimensions_do_not_touch_neighbours():
    """Sub-matrix views: ld > row length.  The cells outside C's view must stay untouched."""
    rng = np.random.default_rng(0)
    M, N, K = 72, 136, 200
    Abig = inp.round_to_dtype(rng.standard_normal((M, K + 24)), inp.DT_BF16)
    Bbig = inp.round_to_dtype(rng.standard_normal((K, N + 8)), inp.DT_BF16)     # k-strided operand
    At, Bt = dev(Abig, torch.bfloat16), dev(Bbig, torch.bfloat16)
    Cbig = torch.full((M, N + 16), -3.0, dtype=torch.float32, device=DEV)
    B.jpp_op_gemm(B.JPP_BF16, M, N, K, At.data_ptr(), K + 24, 0, Bt.data_ptr(), N + 8, 1, Cbig.data_ptr(), N + 16,
                  B.OUT_STORE_F32, None, None, stream())
    torch.cuda.synchronize()
    got = host(Cbig)
    assert rel_l2(got[:, :N], Abig[:, :K] @ Bbig[:, :N]) < 1e-5
    assert np.all(got[:, N:] == -3.0)


def test_gemm_rejects_unsupported_shapes():
    t = torch.zeros(64, 64, dtype=torch.bfloat16, device=DEV)
    f = torch.zeros(64, 64, dtype=torch.float32, device=DEV)
    with pytest.raises(B.JppError) as e:
        B.jpp_op_gemm(B.JPP_BF16, 12, 64, 64, t.data_ptr(), 64, 0, t.data_ptr(), 64, 0, f.data_ptr(), 64,
                      B.OUT_STORE_F32, None, None, stream())
    assert e.value.status == B.JPP_EINVAL
    with pytest.raises(B.JppError):
        B.jpp_op_gemm(B.JPP_BF16, 64, 64, 64, t.data_ptr(), 32, 0, t.data_ptr(), 64, 0, f.data_ptr(), 64,
                      B.OUT_STORE_F32, None, None, stream())
    with pytest.raises(B.JppError):
        B.jpp_op_gemm(B.JPP_BF16, 64, 64, 64, None, 64, 0, t.data_ptr(), 64, 0, f.data_ptr(), 64,
                      B.OUT_STORE_F32, None, None, stream())
    # a row pitch beyond what the 32-bit tile offsets can address is refused, nothing is launched
    with pytest.raises(B.JppError) as e:
        B.jpp_op_gemm(B.JPP_BF16, 64, 64, 64, t.data_ptr(), 1 << 24, 0, t.data_ptr(), 64, 0, f.data_ptr(), 64,
                      B.OUT_STORE_F32, None, None, stream())
    assert e.value.status == B.JPP_EINVAL and "32-bit" in str(e.value)
    with pytest.raises(B.JppError):
        B.jpp_op_gemm_ws(B.JPP_BF16, 64, 64, 64, t.data_ptr(), 64, 0, t.data_ptr(), 64, 0, f.data_ptr(), 64,
                         B.OUT_STORE_F32, None, None, f.data_ptr() + 4, 1024, stream())      # misaligned scratch


@pytest.mark.parametrize("M,N,K", [(5, 3, 7), (130, 70, 33), (64, 64, 16)])
@pytest.mark.parametrize("aks,bks", [(0, 0), (0, 1), (1, 1)])
def test_gemm_f32(M, N, K, aks, bks):
    rng = np.random.default_rng(1)
    A = inp.round_to_dtype(rng.standard_normal((M, K)), inp.DT_F32)
    Bm = inp.round_to_dtype(rng.standard_normal((N, K)), inp.DT_F32)
    bias = inp.round_to_dtype(rng.standard_normal(N), inp.DT_F32)
    At = dev(A.T if aks else A, torch.float32)
    Bt = dev(Bm.T if bks else Bm, torch.float32)
    Cc = torch.ones((M, N), dtype=torch.float32, device=DEV)
    B.jpp_op_gemm(B.JPP_F32, M, N, K, At.data_ptr(), M if aks else K, aks, Bt.data_ptr(), N if bks else K, bks,
                  Cc.data_ptr(), N, B.OUT_ACC_F32, dev(bias, torch.float32).data_ptr(), None, stream())
    torch.cuda.synchronize()
    assert rel_l2(host(Cc), 1.0 + A @ Bm.T + bias[None, :]) < 1e-6


def attention_reference(spec, qkv, dout=None):
    mb, seq, Hq, Hkv, hd = spec.microbatch, spec.seq_len, spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    nq, nkv = Hq * hd, Hkv * hd
    q = qkv[:, :nq].reshape(mb, seq, Hq, hd)
    k = qkv[:, nq:nq + nkv].reshape(mb, seq, Hkv, hd)
    v = qkv[:, nq + nkv:].reshape(mb, seq, Hkv, hd)
    O, P = so.attention_forward(spec, q, k, v)
    if dout is None:
        return O.reshape(mb * seq, nq), None
    dq, dk, dv = so.attention_backward(spec, q, k, v, P, dout.reshape(mb, seq, Hq, hd))
    dqkv = np.concatenate([dq.reshape(mb * seq, nq), dk.reshape(mb * seq, nkv), dv.reshape(mb * seq, nkv)], axis=1)
    return O.reshape(mb * seq, nq), dqkv


ATTN_CASES = [
    # dtype, mb, seq, Hq, Hkv, hd
    (inp.DT_F32, 2, 64, 4, 4, 32), (inp.DT_F32, 1, 37, 3, 1, 24), (inp.DT_BF16, 2, 200, 4, 2, 64),
    (inp.DT_BF16, 2, 256, 4, 4, 128), (inp.DT_BF16, 1, 328, 8, 1, 128), (inp.DT_BF16, 1, 72, 2, 2, 128),
    (inp.DT_BF16, 1, 1, 2, 1, 128),
]


@pytest.mark.parametrize("dtype,mb,seq,Hq,Hkv,hd", ATTN_CASES)
def test_attention_forward_backward(dtype, mb, seq, Hq, Hkv, hd):
    rng = np.random.default_rng(seq + hd)
    spec = so.StageSpec(n_layers=1, d_model=Hq * hd, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=hd, d_ffn=8,
                        seq_len=seq, microbatch=mb)
    T, nqkv = mb * seq, (Hq + 2 * Hkv) * hd
    qkv = inp.round_to_dtype(rng.standard_normal((T, nqkv)), dtype)
    dout = inp.round_to_dtype(rng.standard_normal((T, Hq * hd)), dtype)
    tdt = torch.bfloat16 if dtype == inp.DT_BF16 else torch.float32
    tq, tdo = dev(qkv, tdt), dev(dout, tdt)
    out = torch.zeros((T, Hq * hd), dtype=tdt, device=DEV)
    lse = torch.zeros((mb, Hq, seq), dtype=torch.float32, device=DEV)
    B.jpp_op_attention_fwd(dtype, mb, seq, Hq, Hkv, hd, tq.data_ptr(), out.data_ptr(), lse.data_ptr(), stream())
    dqkv = torch.zeros((T, nqkv), dtype=tdt, device=DEV)
    delta = torch.zeros((mb, Hq, seq), dtype=torch.float32, device=DEV)
    B.jpp_op_attention_bwd(dtype, mb, seq, Hq, Hkv, hd, tq.data_ptr(), out.data_ptr(), lse.data_ptr(),
                           tdo.data_ptr(), dqkv.data_ptr(), delta.data_ptr(), stream())
    torch.cuda.synchronize()
    O, dref = attention_reference(spec, qkv, dout)
    tol = 1e-5 if dtype == inp.DT_F32 else 1e-2
    assert rel_l2(host(out), O) < tol
    # log-sum-exp of the scaled scores, from the definition
    q = qkv[:, :Hq * hd].reshape(mb, seq, Hq, hd)
    k = qkv[:, Hq * hd:(Hq + Hkv) * hd].reshape(mb, seq, Hkv, hd)
    b, h, t = mb - 1, Hq - 1, seq - 1
    s = (k[b, :t + 1, h // (Hq // Hkv)] @ q[b, t, h]) / math.sqrt(hd)
    assert abs(host(lse)[b, h, t] - (s.max() + math.log(np.exp(s - s.max()).sum()))) < (1e-4 if dtype == inp.DT_F32 else 2e-2)
    nq, nkv = Hq * hd, Hkv * hd
    g = host(dqkv)
    for name, sl in (("dq", slice(0, nq)), ("dk", slice(nq, nq + nkv)), ("dv", slice(nq + nkv, nqkv))):
        if np.linalg.norm(dref[:, sl]) == 0.0:      # seq = 1: dS = 0 exactly, so dq = dk = 0
            assert np.abs(g[:, sl]).max() < 1e-5, name
            continue
        assert rel_l2(g[:, sl], dref[:, sl]) < (1e-5 if dtype == inp.DT_F32 else 1.5e-2), name
    # grouped-query shapes on the matrix-core path: the variant that spreads a kv head's query
    # heads over workgroups and sums their dK / dV in head order afterwards
    need = B.jpp_op_attention_bwd_scratch_bytes(dtype, mb, seq, Hq, Hkv, hd)
    assert (need > 0) == (dtype == inp.DT_BF16 and hd == 128 and Hq > Hkv)
    if need:
        scratch = torch.full((need // 4,), float("nan"), dtype=torch.float32, device=DEV)
        dqkv2 = torch.zeros((T, nqkv), dtype=tdt, device=DEV)
        B.jpp_op_attention_bwd_ws(dtype, mb, seq, Hq, Hkv, hd, tq.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                  tdo.data_ptr(), dqkv2.data_ptr(), delta.data_ptr(), scratch.data_ptr(), need, stream())
        torch.cuda.synchronize()
        g2 = host(dqkv2)
        assert np.array_equal(g2[:, :nq], g[:, :nq])            # dQ does not depend on it
        for name, sl in (("dk", slice(nq, nq + nkv)), ("dv", slice(nq + nkv, nqkv))):
            if np.linalg.norm(dref[:, sl]) == 0.0:
                assert np.abs(g2[:, sl]).max() < 1e-5, name
                continue
            assert rel_l2(g2[:, sl], dref[:, sl]) < 1.5e-2, name
            assert rel_l2(g2[:, sl], g[:, sl]) < 8e-3, name     # same sums, another association, bf16 rounding


@pytest.mark.parametrize("dtype", [inp.DT_F32, inp.DT_BF16])
@pytest.mark.parametrize("norm", [inp.NORM_LAYERNORM, inp.NORM_RMSNORM])
@pytest.mark.parametrize("rows,d", [(5, 72), (300, 2048), (64, 12288), (2048, 12288),
                                    # rows of 1024 chunks and more take the 512-thread backward form:
                                    # exact multiples, ragged last chunks per thread, no added tensor (odd rows)
                                    (40, 8192), (33, 8200), (300, 6144), (17, 12280), (600, 4096)])
def test_norm_forward_backward(dtype, norm, rows, d):
    if dtype == inp.DT_F32 and d > 8192:
        pytest.skip("fp32 rows are limited to 8192 columns")
    _norm_case(dtype, norm, rows, d, rows % 2 == 0)


@pytest.mark.parametrize("norm", [inp.NORM_LAYERNORM, inp.NORM_RMSNORM])
@pytest.mark.parametrize("rows,d,with_add", [(1024, 2048, True), (1024, 2048, False), (2048, 2048, True),
                                             (512, 4096, True), (512, 4096, False), (1536, 4096, True)])
def test_norm_backward_rows_that_fill_the_workgroups_exactly(norm, rows, d, with_add):
    """bf16 rows of exactly 256 or 512 chunks, in row counts that give every workgroup only full
    turns (four or two rows at a time): the backward forms without predicates, with and without
    the added tensor."""
    _norm_case(inp.DT_BF16, norm, rows, d, with_add)


def _norm_case(dtype, norm, rows, d, with_add):
    rng = np.random.default_rng(rows + d)
    spec = so.StageSpec(n_layers=1, d_model=d, n_q_heads=1, n_kv_heads=1, head_dim=8, d_ffn=8, seq_len=1,
                        microbatch=1, norm=norm)
    x = inp.round_to_dtype(rng.standard_normal((rows, d)) * 1.5 + 0.3, dtype)
    g = inp.round_to_dtype(1 + 0.1 * rng.standard_normal(d), dtype)
    b = inp.round_to_dtype(0.1 * rng.standard_normal(d), dtype)
    dy = inp.round_to_dtype(rng.standard_normal((rows, d)), dtype)
    add = inp.round_to_dtype(rng.standard_normal((rows, d)), dtype)
    tdt = torch.bfloat16 if dtype == inp.DT_BF16 else torch.float32
    tx, tg, tb, tdy, tadd = (dev(a, tdt) for a in (x, g, b, dy, add))
    y = torch.zeros_like(tx)
    stats = torch.zeros(2 * rows, dtype=torch.float32, device=DEV)
    B.jpp_op_norm_fwd(dtype, norm, rows, d, 1e-5, tx.data_ptr(), tg.data_ptr(), tb.data_ptr(), y.data_ptr(),
                      stats.data_ptr(), stream())
    dx = torch.zeros_like(tx)
    gg = torch.ones(d, dtype=torch.float32, device=DEV)
    gb = torch.ones(d, dtype=torch.float32, device=DEV)
    part = torch.zeros(B.jpp_op_colreduce_scratch(rows, d), dtype=torch.float32, device=DEV)
    B.jpp_op_norm_bwd(dtype, norm, rows, d, tx.data_ptr(), tg.data_ptr(), stats.data_ptr(), tdy.data_ptr(),
                      tadd.data_ptr() if with_add else None, dx.data_ptr(), gg.data_ptr(), gb.data_ptr(),
                      part.data_ptr(), stream())
    torch.cuda.synchronize()
    if not with_add:
        add = 0.0
    yr, xhat, rstd = so.norm_forward(spec, x, g, b if norm == inp.NORM_LAYERNORM else 0.0)
    dxr, dgr, dbr = so.norm_backward(spec, dy, xhat, rstd, g)
    tol = 1e-5 if dtype == inp.DT_F32 else 6e-3
    assert rel_l2(host(y), yr) < tol
    assert rel_l2(host(dx), dxr + add) < tol
    assert rel_l2(host(gg), 1 + dgr) < 1e-5
    if norm == inp.NORM_LAYERNORM:
        assert rel_l2(host(gb), 1 + dbr) < 1e-5
    else:
        assert np.all(host(gb) == 1.0)


@pytest.mark.parametrize("dtype", [inp.DT_F32, inp.DT_BF16])
@pytest.mark.parametrize("act", [inp.ACT_GELU, inp.ACT_GELU_TANH, inp.ACT_SWIGLU])
@pytest.mark.parametrize("rows,f", [(77, 520), (9, 4104)])   # ragged row groups; several column blocks, ragged last
def test_activation_forward_backward(dtype, act, rows, f):
    rng = np.random.default_rng(act)
    spec = so.StageSpec(n_layers=1, d_model=8, n_q_heads=1, n_kv_heads=1, head_dim=8, d_ffn=f, seq_len=1,
                        microbatch=1, act=act)
    f1 = 2 * f if act == inp.ACT_SWIGLU else f
    h = inp.round_to_dtype(rng.standard_normal((rows, f1)) * 2, dtype)
    da = inp.round_to_dtype(rng.standard_normal((rows, f)), dtype)
    tdt = torch.bfloat16 if dtype == inp.DT_BF16 else torch.float32
    th, tda = dev(h, tdt), dev(da, tdt)
    a = torch.zeros((rows, f), dtype=tdt, device=DEV)
    dh = torch.zeros((rows, f1), dtype=tdt, device=DEV)
    B.jpp_op_act_fwd(dtype, act, rows, f, th.data_ptr(), a.data_ptr(), stream())
    B.jpp_op_act_bwd(dtype, act, rows, f, th.data_ptr(), tda.data_ptr(), dh.data_ptr(), stream())
    torch.cuda.synchronize()
    tol = 2e-6 if dtype == inp.DT_F32 else 4e-3
    assert rel_l2(host(a), so.act_forward(spec, h)) < tol
    assert rel_l2(host(dh), so.act_backward(spec, h, da)) < tol


@pytest.mark.parametrize("dtype,rows,vocab", [(inp.DT_F32, 7, 1000), (inp.DT_F32, 5, 1001), (inp.DT_F32, 3, 6),
                                              (inp.DT_BF16, 9, 5024), (inp.DT_BF16, 4, 8), (inp.DT_BF16, 2, 70000),
                                              (inp.DT_BF16, 3, 2048), (inp.DT_F32, 3, 2052), (inp.DT_BF16, 2, 51200),
                                              (inp.DT_BF16, 3, 51204), (inp.DT_F32, 2, 60000), (inp.DT_BF16, 2, 65536),
                                              (inp.DT_BF16, 4096, 50304)])
def test_cross_entropy(dtype, rows, vocab):
    """Loss, per-row losses and dz against the float64 definition; vocabularies that take the
    register-resident kernels (a multiple of 4: up to 51200 in 512 threads, up to 65536 in 1024,
    with the last chunk of a thread full and ragged) and ones that do not, and the
    C5 head's own shape (4096 x 50304: 256 sampled rows for dz, every row's loss)."""
    g = torch.Generator(device=DEV)
    g.manual_seed(rows + vocab)
    z = torch.randn((rows, vocab), generator=g, device=DEV) * 3
    tg = torch.randint(0, vocab, (rows,), generator=g, device=DEV, dtype=torch.int32)
    tdt = torch.bfloat16 if dtype == inp.DT_BF16 else torch.float32
    dz = torch.full((rows, vocab), float("nan"), dtype=tdt, device=DEV)
    rl = torch.zeros(rows, dtype=torch.float32, device=DEV)
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    B.jpp_op_cross_entropy(dtype, rows, vocab, z.data_ptr(), tg.data_ptr(), dz.data_ptr(), rl.data_ptr(),
                           loss.data_ptr(), stream())
    torch.cuda.synchronize()
    assert bool(torch.isfinite(dz.float()).all())
    rng = np.random.default_rng(3)
    pick = np.arange(rows) if rows <= 256 else np.unique(np.concatenate([rng.integers(0, rows, 254), [0, rows - 1]]))
    idx = torch.from_numpy(pick).to(DEV)
    zh = host(z[idx])
    th = tg[idx].cpu().numpy()
    zs = zh - zh.max(axis=1, keepdims=True)
    logp = zs - np.log(np.exp(zs).sum(axis=1, keepdims=True))
    want_rl = -logp[np.arange(len(pick)), th]
    want_dz = np.exp(logp)
    want_dz[np.arange(len(pick)), th] -= 1.0
    want_dz /= rows
    assert rel_l2(host(rl[idx]), want_rl) < 1e-6
    assert rel_l2(host(dz[idx]), want_dz) < (1e-5 if dtype == inp.DT_F32 else 4e-3)
    assert abs(float(loss[0]) - float(rl.double().mean())) <= 1e-6 * abs(float(loss[0]))


# ------------------------------------------------------------------ full benchmark shapes

@pytest.mark.parametrize("act", [inp.ACT_GELU, inp.ACT_SWIGLU])
def test_activation_full_shape_sampled_rows(act):
    """The element-wise kernels at the C4 FFN shape (2048 x 49152, bf16): 128 sampled rows plus
    the first and the last against the oracle; rows between them must not be left untouched."""
    rows, f = 2048, 49152
    f1 = 2 * f if act == inp.ACT_SWIGLU else f
    g = torch.Generator(device=DEV)
    g.manual_seed(17 + act)
    th = (torch.randn((rows, f1), generator=g, device=DEV) * 2).to(torch.bfloat16)
    tda = torch.randn((rows, f), generator=g, device=DEV).to(torch.bfloat16)
    a = torch.full((rows, f), float("nan"), dtype=torch.bfloat16, device=DEV)
    dh = torch.full((rows, f1), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.jpp_op_act_fwd(inp.DT_BF16, act, rows, f, th.data_ptr(), a.data_ptr(), stream())
    B.jpp_op_act_bwd(inp.DT_BF16, act, rows, f, th.data_ptr(), tda.data_ptr(), dh.data_ptr(), stream())
    torch.cuda.synchronize()
    assert bool(torch.isfinite(a.float()).all()) and bool(torch.isfinite(dh.float()).all())
    rng = np.random.default_rng(5)
    pick = np.unique(np.concatenate([rng.integers(0, rows, 128), [0, rows - 1]]))
    idx = torch.from_numpy(pick).to(DEV)
    spec = so.StageSpec(n_layers=1, d_model=8, n_q_heads=1, n_kv_heads=1, head_dim=8, d_ffn=f, seq_len=1,
                        microbatch=1, act=act)
    h, da = host(th[idx]), host(tda[idx])
    assert rel_l2(host(a[idx]), so.act_forward(spec, h)) < 4e-3
    assert rel_l2(host(dh[idx]), so.act_backward(spec, h, da)) < 4e-3


FULL_GEMMS = [
    # the GPT-3-shaped layer's GEMMs at T = 2048 tokens: (M, N, K, a_kstrided, b_kstrided, out_mode)
    ("qkv fwd", 2048, 36864, 12288, 0, 0, B.OUT_STORE),
    ("ffn-down dgrad", 2048, 49152, 12288, 0, 1, B.OUT_STORE),
    ("ffn-up wgrad", 49152, 12288, 2048, 1, 1, B.OUT_ACC_F32),
    ("lm-head fwd", 4096, 50304, 4096, 0, 0, B.OUT_STORE_F32),
    # weight gradients over a group of 8 microbatches (K = 8 * 2048)
    ("ffn-down wgrad, group of 8", 12288, 49152, 16384, 1, 1, B.OUT_ACC_F32),
    ("qkv wgrad, group of 4", 36864, 12288, 8192, 1, 1, B.OUT_ACC_F32),
]


@pytest.mark.parametrize("name,M,N,K,aks,bks,mode", FULL_GEMMS)
def test_gemm_full_shape_sampled_entries(name, M, N, K, aks, bks, mode):
    """At the benchmark's sizes the outputs are checked on sampled entries (random ones plus
    the corners and tile edges), each against a float64 dot product of the kernel's inputs."""
    g = torch.Generator(device=DEV)
    g.manual_seed(M + N + K)
    A = torch.randn((K, M) if aks else (M, K), generator=g, device=DEV).to(torch.bfloat16)
    Bm = (torch.randn((K, N) if bks else (N, K), generator=g, device=DEV) * 0.02).to(torch.bfloat16)
    if mode == B.OUT_STORE:
        Cc = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    else:
        Cc = torch.ones((M, N), dtype=torch.float32, device=DEV)
    B.jpp_op_gemm(B.JPP_BF16, M, N, K, A.data_ptr(), M if aks else K, aks, Bm.data_ptr(), N if bks else K, bks,
                  Cc.data_ptr(), N, mode, None, None, stream())
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    ms = np.concatenate([rng.integers(0, M, 4096), [0, 0, M - 1, M - 1, 255, 256, M - 256, M - 257]])
    ns = np.concatenate([rng.integers(0, N, 4096), [0, N - 1, 0, N - 1, 255, 256, N - 256, N - 257]])
    mi, ni = torch.from_numpy(ms).to(DEV), torch.from_numpy(ns).to(DEV)
    # the sampled operand rows are brought to the host; the reference is a float64 dot product there
    a_rows = (A[:, mi].T if aks else A[mi, :]).float().cpu().numpy().astype(np.float64)
    b_rows = (Bm[:, ni].T if bks else Bm[ni, :]).float().cpu().numpy().astype(np.float64)
    ref = np.einsum("sk,sk->s", a_rows, b_rows)
    got = Cc[mi, ni].double().cpu().numpy()
    if mode == B.OUT_ACC_F32:
        ref = ref + 1.0
    tol = 4e-3 if mode == B.OUT_STORE else 1e-5
    assert rel_l2(got, ref) < tol, name
    assert np.all(np.isfinite(got))


@pytest.mark.parametrize("M,N", [(49152, 12288), (12288, 49152), (36864, 12288), (12288, 12288), (12288 + 256, 12288),
                                 (4096, 8192)])
def test_accumulating_gemm_adds_to_every_tile_exactly_once(M, N):
    """The workgroup-to-tile maps (one of them only used when both tile counts are multiples
    of 16) must be bijections: with all-ones operands and K = 64 every element of an
    accumulating GEMM grows by exactly 64, twice in a row."""
    K = 64
    A = torch.ones((K, M), dtype=torch.bfloat16, device=DEV)
    Bm = torch.ones((K, N), dtype=torch.bfloat16, device=DEV)
    Cc = torch.full((M, N), 3.0, dtype=torch.float32, device=DEV)
    for rep in (1, 2):
        B.jpp_op_gemm(B.JPP_BF16, M, N, K, A.data_ptr(), M, 1, Bm.data_ptr(), N, 1, Cc.data_ptr(), N, B.OUT_ACC_F32,
                      None, None, stream())
        torch.cuda.synchronize()
        assert bool((Cc == 3.0 + 64.0 * rep).all()), (M, N, rep)


FULL_ATTENTION = [
    # name, mb, seq, Hq, Hkv, sampled kv heads (with their whole query groups)
    ("C4 layer", 1, 2048, 96, 96, [0, 50, 95]),
    ("C3 layer", 1, 4096, 64, 8, [5]),
    ("C5 layer", 2, 2048, 32, 32, [31]),
]


@pytest.mark.parametrize("name,mb,seq,Hq,Hkv,kv_heads", FULL_ATTENTION)
def test_attention_full_shape_sampled_heads(name, mb, seq, Hq, Hkv, kv_heads):
    """The benchmark's attention shapes: the kernels run on every head; the float64 definition is
    evaluated for a few kv heads together with all query heads that read them."""
    hd, grp = 128, Hq // Hkv
    g = torch.Generator(device=DEV)
    g.manual_seed(seq + Hq)
    T, nq, nkv = mb * seq, Hq * hd, Hkv * hd
    tq = torch.randn((T, nq + 2 * nkv), generator=g, device=DEV).to(torch.bfloat16)
    tdo = torch.randn((T, nq), generator=g, device=DEV).to(torch.bfloat16)
    out = torch.zeros((T, nq), dtype=torch.bfloat16, device=DEV)
    lse = torch.zeros((mb, Hq, seq), dtype=torch.float32, device=DEV)
    dqkv = torch.zeros_like(tq)
    delta = torch.zeros((mb, Hq, seq), dtype=torch.float32, device=DEV)
    B.jpp_op_attention_fwd(inp.DT_BF16, mb, seq, Hq, Hkv, hd, tq.data_ptr(), out.data_ptr(), lse.data_ptr(), stream())
    # as the executor calls it: with the scratch a grouped-query shape asks for
    need = B.jpp_op_attention_bwd_scratch_bytes(inp.DT_BF16, mb, seq, Hq, Hkv, hd)
    scratch = torch.full((max(need // 4, 4),), float("nan"), dtype=torch.float32, device=DEV)
    B.jpp_op_attention_bwd_ws(inp.DT_BF16, mb, seq, Hq, Hkv, hd, tq.data_ptr(), out.data_ptr(), lse.data_ptr(),
                              tdo.data_ptr(), dqkv.data_ptr(), delta.data_ptr(), scratch.data_ptr(), need, stream())
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out.float()).all()) and bool(torch.isfinite(dqkv.float()).all())
    for kv in kv_heads:
        qcols = slice(kv * grp * hd, (kv + 1) * grp * hd)
        kcols = slice(nq + kv * hd, nq + (kv + 1) * hd)
        vcols = slice(nq + nkv + kv * hd, nq + nkv + (kv + 1) * hd)
        spec = so.StageSpec(n_layers=1, d_model=grp * hd, n_q_heads=grp, n_kv_heads=1, head_dim=hd, d_ffn=8,
                            seq_len=seq, microbatch=mb)
        q = host(tq[:, qcols]).reshape(mb, seq, grp, hd)
        k = host(tq[:, kcols]).reshape(mb, seq, 1, hd)
        v = host(tq[:, vcols]).reshape(mb, seq, 1, hd)
        O, P = so.attention_forward(spec, q, k, v)
        dq, dk, dv = so.attention_backward(spec, q, k, v, P, host(tdo[:, qcols]).reshape(mb, seq, grp, hd))
        assert rel_l2(host(out[:, qcols]), O.reshape(T, grp * hd)) < 1e-2, (name, kv)
        assert rel_l2(host(dqkv[:, qcols]), dq.reshape(T, grp * hd)) < 1e-2, (name, kv)
        assert rel_l2(host(dqkv[:, kcols]), dk.reshape(T, hd)) < 1e-2, (name, kv)
        assert rel_l2(host(dqkv[:, vcols]), dv.reshape(T, hd)) < 1e-2, (name, kv)
