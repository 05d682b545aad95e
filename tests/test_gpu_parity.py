"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Codes, scales, row sums and the int32 contract value A4 must agree bit for bit;
fp32 outputs within 1e-6 relative; the bf16 backward within 2e-2 relative Frobenius."""
import numpy as np
import pytest
import torch

import oracle
from paper_1909_05840_amd import workloads as wl

pytestmark = pytest.mark.gpu
BITS = (2, 3, 4, 8)
CLIP = 6.0
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


def gpu_quantize(qb, W, bits, G):
    Wd = W.to(DEV)
    packed, h, m, rs = qb.qb_quantize_groupwise(Wd, bits, G)
    codes = qb.qb_unpack_codes(packed, W.shape[0], W.shape[1], bits)
    torch.cuda.synchronize()
    return packed, h, m, rs, codes


def check_quantize(qb, W, bits, G):
    say("quantize", tuple(W.shape), "bits", bits, "G", G)
    packed, h, m, rs, codes = gpu_quantize(qb, W, bits, G)
    oc, oh, om, ors = oracle.quantize_groupwise(W.numpy(), bits, G)
    assert (codes.cpu().numpy() == oc).all()
    assert (h.cpu().numpy().view(np.uint32) == oh.view(np.uint32)).all()
    assert (m.cpu().numpy().view(np.uint32) == om.view(np.uint32)).all()
    assert (rs.cpu().numpy() == ors).all()
    assert packed.numel() == qb.qb_packed_nbytes(W.shape[0], W.shape[1], bits)
    return packed, h, rs, oc, oh


# ---- weights ---------------------------------------------------------------------------------
@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", [(768, 768, 128), (2304, 768, 128), (2304, 768, 384), (3072, 768, 128),
                                   (768, 3072, 128), (1024, 4096, 128), (4096, 1024, 128)])
def test_quantize_bert_shapes(qb, bits, shape):
    N, K, G = shape
    check_quantize(qb, wl.weight(N, K, seed=N + K + bits), bits, G)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", [(768, 768, 1), (768, 768, 12), (768, 768, 24), (768, 768, 768), (6, 64, 1),
                                   (6, 64, 6), (40, 192, 8), (100, 128, 4), (33, 64, 33), (1030, 64, 1)])
def test_quantize_group_special_cases_and_ragged(qb, bits, shape):
    N, K, G = shape
    check_quantize(qb, wl.weight_uniform(N, K, seed=7 * N + K + bits), bits, G)


def test_quantize_zero_group_ties_and_extremes(qb):
    W = wl.weight_uniform(64, 256, seed=5)
    W[0:8] = 0.0                      # an all-zero group
    h = 0.25
    for bits in BITS:
        L = 2 ** bits - 1
        Wt = W.clone()
        ties = torch.tensor([h * (2 * j + 1 - L) for j in range(L)], dtype=torch.float32)
        Wt[8:16] = 0.0
        Wt[8, 0], Wt[8, 1] = -h * L, h * L
        Wt[9, :L] = ties              # exact half-way points: must go to the even code
        check_quantize(qb, Wt, bits, 8)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", [(768, 768, 128), (2304, 768, 128), (768, 3072, 128), (96, 64, 96), (6, 64, 1), (768, 768, 1)])
def test_quantize_given_clipped_range(qb, bits, shape):
    """Ranges given by the caller: half of each group's max-abs (about the outer weights are clamped), then the
    max-abs itself (must reproduce the plain call), then zero."""
    N, K, G = shape
    say("quantize clip", shape, "bits", bits)
    W = wl.weight_uniform(N, K, seed=3 * N + K + bits, lo=-0.1, hi=0.1)
    _, _, om, _ = oracle.quantize_groupwise(W.numpy(), bits, G)
    for scale in (0.5, 1.0, 0.0):
        m_in = (om * np.float32(scale)).astype(np.float32)
        packed, h, rs = qb.qb_quantize_groupwise_clip(W.to(DEV), bits, torch.from_numpy(m_in).to(DEV))
        codes = qb.qb_unpack_codes(packed, N, K, bits)
        torch.cuda.synchronize()
        oc, oh, ors = oracle.quantize_groupwise_clip(W.numpy(), bits, m_in)
        assert (codes.cpu().numpy() == oc).all()
        assert (h.cpu().numpy().view(np.uint32) == oh.view(np.uint32)).all()
        assert (rs.cpu().numpy() == ors).all()
        if scale == 0.5:
            L = 2 ** bits - 1
            assert (oc == 0).any() and (oc == L).any()


def test_quantize_batched_matches_single_calls(qb):
    """Configuration 4 style: 12 layers x 4 linears, each layer at its own bit-width, in batched launches
    (more jobs than one launch holds, mixed bits, one job with groups too large for the fused path)."""
    bits_list = wl.layer_bits(12, seed=wl.config_seed(3, 0))
    jobs, singles = [], []
    for layer in range(5):
        for i, (_, N, K) in enumerate(wl.BERT_BASE_LINEARS):
            W = wl.weight(N, K, seed=100 * layer + i).to(DEV)
            jobs.append({"W": W, "bits": bits_list[layer], "groups": 128})
    jobs.append({"W": wl.weight_uniform(768, 768, seed=9).to(DEV), "bits": 3, "groups": 1})  # two-pass job
    say("batched quantize", len(jobs), "jobs")
    outs = qb.qb_quantize_groupwise_batched(jobs)
    for j, (packed, h, m, rs) in zip(jobs, outs):
        p1, h1, m1, r1 = qb.qb_quantize_groupwise(j["W"], j["bits"], j["groups"])
        torch.cuda.synchronize()
        assert torch.equal(packed, p1) and torch.equal(h, h1) and torch.equal(m, m1) and torch.equal(rs, r1)
    # and against the oracle for two of them
    for idx in (0, 7):
        j = jobs[idx]
        N, K = j["W"].shape
        oc, oh, om, ors = oracle.quantize_groupwise(j["W"].cpu().numpy(), j["bits"], j["groups"])
        codes = qb.qb_unpack_codes(outs[idx][0], N, K, j["bits"])
        assert (codes.cpu().numpy() == oc).all() and (outs[idx][3].cpu().numpy() == ors).all()


def test_hip_graph_replays_match_eager(qb):
    """The calls only enqueue kernels, so a captured graph must give the eager result on every replay."""
    T, N, K, G, bits = 512, 768, 768, 128, 4
    W = wl.weight(N, K, seed=21).to(DEV)
    X = wl.activation(T, K, seed=22).to(DEV)
    packed, h, m, rs_w = qb.qb_quantize_groupwise(W, bits, G)
    Xq, rs_x = qb.qb_quantize_act(X, CLIP)
    Y_eager = qb.qb_qlinear_fwd(Xq, rs_x, CLIP, packed, h, rs_w, bits, G, N).clone()
    Yq_eager, rsy_eager = [t.clone() for t in qb.qb_qlinear_fwd_q8(Xq, rs_x, CLIP, packed, h, rs_w, bits, G, N, 2.0)]
    p_eager = packed.clone()
    torch.cuda.synchronize()
    Y = torch.empty_like(Y_eager)
    Yq, rs_y = torch.empty_like(Yq_eager), torch.empty_like(rsy_eager)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            qb.qb_quantize_groupwise_batched([{"W": W, "bits": bits, "groups": G, "packed": packed, "h": h, "m": m,
                                               "rs_w": rs_w}])
            qb.qb_quantize_act(X, CLIP, Xq, rs_x)
            qb.qb_qlinear_fwd(Xq, rs_x, CLIP, packed, h, rs_w, bits, G, N, Y=Y)
            qb.qb_qlinear_fwd_q8(Xq, rs_x, CLIP, packed, h, rs_w, bits, G, N, 2.0, Yq=Yq, rs_y=rs_y)
        for rep in range(4):
            Y.zero_()
            packed.zero_()
            Yq.zero_()
            rs_y.fill_(12345)   # the call clears the row sums itself, on every replay
            stream.synchronize()
            g.replay()
            stream.synchronize()
            assert torch.equal(Y, Y_eager) and torch.equal(packed, p_eager), rep
            assert torch.equal(Yq, Yq_eager) and torch.equal(rs_y, rsy_eager), rep
            # eager work of the program between replays
            Y2 = qb.qb_qlinear_fwd(Xq, rs_x, CLIP, packed, h, rs_w, bits, G, N)
            stream.synchronize()
            assert torch.equal(Y2, Y_eager)


def test_hip_graph_replays_of_range_variants_and_backward(qb):
    """The entry points that clear or initialise device scratch themselves (per-tensor dynamic range, asymmetric ranges)
    and the backward, captured in one graph: every replay, with the outputs and scratch overwritten and eager work in
    between, gives the eager result."""
    T, N, K, G, bits = 640, 768, 768, 128, 3
    W = wl.weight(N, K, seed=31).abs().contiguous().to(DEV)
    X = wl.activation(T, K, seed=32).to(DEV)
    dY = wl.grad_output_bf16(T, N, seed=33).to(DEV)
    clip = 1.5
    e_xq, e_rs, e_hx, e_c = [t.clone() for t in qb.qb_quantize_act_dyn_tensor(X)]
    e_p, e_d, e_q0, e_rw = [t.clone() for t in qb.qb_quantize_groupwise_asym(W, bits, G)]
    Xq, rs_x = qb.qb_quantize_act(X, clip)
    e_Y = qb.qb_qlinear_fwd_asym(Xq, rs_x, clip, e_p, e_d, e_q0, e_rw, bits, G, N).clone()
    e_dX, e_dW = [t.clone() for t in qb.qb_qlinear_bwd_ste_asym(dY, Xq, clip, e_p, e_d, e_q0, bits, G)]
    e_mX, _ = qb.qb_qlinear_bwd_ste_masked(dY, Xq, clip, e_p, e_d, bits, G, X=X, want_dw=False)
    e_mX = e_mX.clone()
    torch.cuda.synchronize()
    xq, rs, hx, c = [torch.empty_like(t) for t in (e_xq, e_rs, e_hx, e_c)]
    p, d, q0, rw = [torch.empty_like(t) for t in (e_p, e_d, e_q0, e_rw)]
    Y, dX, dW, mX = [torch.empty_like(t) for t in (e_Y, e_dX, e_dW, e_mX)]
    ws = torch.empty(qb.qb_bwd_workspace_nbytes(T, N, K), dtype=torch.uint8, device=DEV)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            qb.qb_quantize_act_dyn_tensor(X, xq, rs, hx, c)
            qb.qb_quantize_groupwise_asym(W, bits, G, p, d, q0, rw)
            qb.qb_qlinear_fwd_asym(Xq, rs_x, clip, p, d, q0, rw, bits, G, N, Y=Y)
            qb.qb_qlinear_bwd_ste_asym(dY, Xq, clip, p, d, q0, bits, G, dX=dX, dW=dW, workspace=ws)
            qb.qb_qlinear_bwd_ste_masked(dY, Xq, clip, p, d, bits, G, X=X, want_dw=False, dX=mX, workspace=ws)
        for rep in range(3):
            for t in (xq, rs, hx, p, rw, Y, dX, dW, mX, ws):
                t.zero_()
            c.fill_(1.0e30)     # the reduction's scratch: cleared by the call on every replay
            d.fill_(7.0)
            q0.fill_(-7.0)
            stream.synchronize()
            g.replay()
            stream.synchronize()
            for a, b in ((xq, e_xq), (rs, e_rs), (hx, e_hx), (c, e_c), (p, e_p), (d, e_d), (q0, e_q0), (rw, e_rw), (Y, e_Y),
                         (dX, e_dX), (dW, e_dW), (mX, e_mX)):
                assert torch.equal(a, b), rep
            Y2 = qb.qb_qlinear_fwd_asym(Xq, rs_x, clip, e_p, e_d, e_q0, e_rw, bits, G, N)   # eager work between replays
            stream.synchronize()
            assert torch.equal(Y2, e_Y)


# ---- activations ---------------------------------------------------------------------------------
@pytest.mark.parametrize("shape", [(1024, 768), (4096, 768), (4096, 3072), (1, 64), (1023, 768), (7, 1024), (130, 4096)])
def test_quantize_act(qb, shape):
    T, K = shape
    say("act", shape)
    X = wl.activation(T, K, seed=T + K)
    X[0, :8] = torch.tensor([0.0, -0.0, 6.0, -6.0, 100.0, -100.0, float("inf"), float("-inf")])
    Xq, rs = qb.qb_quantize_act(X.to(DEV), CLIP)
    oq, ors = oracle.quantize_act(X.numpy(), CLIP)
    assert (Xq.cpu().numpy() == oq).all()
    assert (rs.cpu().numpy() == ors).all()


# ---- forward ---------------------------------------------------------------------------------------
def run_fwd(qb, W, X, bits, G, bias=None):
    N, K = W.shape
    packed, h, rs_w, oc, oh = check_quantize(qb, W, bits, G)
    Xq, rs_x = qb.qb_quantize_act(X.to(DEV), CLIP)
    Y, A4 = qb.qb_qlinear_fwd(Xq, rs_x, CLIP, packed, h, rs_w, bits, G, N,
                              bias=None if bias is None else bias.to(DEV), want_a4=True)
    torch.cuda.synchronize()
    oq, _ = oracle.quantize_act(X.numpy(), CLIP)
    assert (Xq.cpu().numpy() == oq).all()
    return Y.cpu().numpy(), A4.cpu().numpy(), oq, oc, oh


def assert_rel(Y, Yo, tol=1e-6):
    err = np.abs(Y.astype(np.float64) - Yo.astype(np.float64))
    assert (err <= tol * np.abs(Yo.astype(np.float64))).all(), float((err / np.maximum(np.abs(Yo), 1e-30)).max())


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", [(300, 160, 192, 8), (257, 96, 64, 96), (1, 32, 64, 1), (129, 130, 320, 10),
                                   (513, 768, 768, 128), (64, 6, 128, 6), (100, 96, 2048, 96), (1700, 1536, 192, 128)])
def test_forward_full_compare(qb, bits, shape):
    """Several tiles and ragged tails in T, N; full element-by-element comparison."""
    T, N, K, G = shape
    say("fwd full", shape, "bits", bits)
    W = wl.weight_uniform(N, K, seed=11 * N + K + bits, lo=-0.1, hi=0.1)
    X = wl.activation(T, K, seed=T + K + bits)
    Y, A4, oq, oc, oh = run_fwd(qb, W, X, bits, G)
    Yo, A4o, _ = oracle.qlinear_fwd(oq, CLIP, oc, oh, bits, openmp=True)
    assert (A4 == A4o).all()
    assert_rel(Y, Yo)
    assert (Y[A4o == 0] == 0).all()


@pytest.mark.parametrize("bits", BITS)
def test_forward_maximum_K_and_extreme_codes(qb, bits):
    """The longest contraction the ABI accepts (K = 32768) with every operand at an end of its range: |A4| reaches
    255 * L * K (2.13e9 at 8 bits, just inside int32, where the kernel's intermediate 4*acc touches 2^31)."""
    T, N, K, G = 96, 64, 32768, 32
    say("fwd max K", (T, N, K), "bits", bits)
    W = torch.full((N, K), 0.1)
    W[1::2] = -0.1                      # groups of two rows: codes L and 0
    W[5, ::3] = 0.02
    X = torch.full((T, K), 6.0)
    X[1::3] = -6.0                      # x' = 127 and -128
    X[2::3] = wl.activation(T, K, seed=5)[2::3]
    Y, A4, oq, oc, oh = run_fwd(qb, W, X, bits, G)
    Yo, A4o, _ = oracle.qlinear_fwd(oq, CLIP, oc, oh, bits, openmp=True)
    assert int(np.abs(A4o.astype(np.int64)).max()) == 255 * (2 ** bits - 1) * K   # 2.13e9 at 8 bits
    assert (A4 == A4o).all()
    assert_rel(Y, Yo)


@pytest.mark.parametrize("bits", (3, 8))
def test_forward_maximum_K_role_split_kernels(qb, bits):
    """The same extremes through the 128x96 role-split kernel (4096 x 768 outputs): sampled positions against the
    oracle, and every output whose token row and neuron row are constant against the closed form
    A4 = K * (2x'+1) * (2c'+1)."""
    T, N, K, G = 4096, 768, 32768, 128
    say("fwd max K role-split", (T, N, K), "bits", bits)
    L = 2 ** bits - 1
    W = torch.full((N, K), 0.1)
    W[1::2] = -0.1
    W[4::6, ::5] = 0.03                 # some rows with mixed codes
    X = torch.full((T, K), 6.0)
    X[1::3] = -6.0
    X[2::3, ::2] = 0.7
    packed, h, m, rs_w = qb.qb_quantize_groupwise(W.to(DEV), bits, G)
    Xq, rs_x = qb.qb_quantize_act(X.to(DEV), CLIP)
    Y, A4 = qb.qb_qlinear_fwd(Xq, rs_x, CLIP, packed, h, rs_w, bits, G, N, want_a4=True)
    torch.cuda.synchronize()
    A4 = A4.cpu().numpy()
    oc, oh, _, _ = oracle.quantize_groupwise(W.numpy(), bits, G)
    oq, _ = oracle.quantize_act(X.numpy(), CLIP)
    assert (qb.qb_unpack_codes(packed, N, K, bits).cpu().numpy() == oc).all() and (Xq.cpu().numpy() == oq).all()
    r = np.random.default_rng(bits)
    ts, ns = r.integers(0, T, 600), r.integers(0, N, 600)
    Ys, A4s = oracle.qlinear_fwd_sampled(oq, CLIP, oc, oh, bits, ts, ns)
    assert (A4[ts, ns] == A4s).all()
    assert_rel(Y.cpu().numpy()[ts, ns], Ys)
    xrow = np.where((oq == oq[:, :1]).all(axis=1))[0]          # constant token rows
    wrow = np.where((oc == oc[:, :1]).all(axis=1))[0]          # constant neuron rows
    assert len(xrow) > T // 2 and len(wrow) > N // 2
    fx = 2 * oq[xrow, 0].astype(np.int64) + 1
    fw = 2 * oc[wrow, 0].astype(np.int64) - L
    assert (A4[np.ix_(xrow, wrow)] == K * fx[:, None] * fw[None, :]).all()
    assert int(np.abs(A4.astype(np.int64)).max()) == 255 * L * K


def test_forward_config1_and_bias(qb):
    """Configuration 1: one BERT-base Q projection, 4-bit, 128 groups, T = 1024, seed 0."""
    W = wl.weight(768, 768, seed=wl.config_seed(0, 0))
    X = wl.activation(1024, 768, seed=wl.config_seed(0, 1))
    Y, A4, oq, oc, oh = run_fwd(qb, W, X, 4, 128)
    Yo, A4o, _ = oracle.qlinear_fwd(oq, CLIP, oc, oh, 4, openmp=True)
    assert (A4 == A4o).all()
    assert_rel(Y, Yo)
    bias = wl.activation(1, 768, seed=3)[0].contiguous()
    Yb, A4b, _, _, _ = run_fwd(qb, W, X, 4, 128, bias=bias)
    assert (A4b == A4o).all()
    Yob, _, _ = oracle.qlinear_fwd(oq, CLIP, oc, oh, 4, bias=bias.numpy(), openmp=True)
    assert np.abs(Yb - Yob).max() <= 1e-6 * max(np.abs(Yo).max(), np.abs(bias.numpy()).max())


def sampled_fwd_check(qb, T, N, K, G, bits, seed, n_samples=4096):
    say("fwd sampled", (T, N, K, G), "bits", bits)
    W = wl.weight(N, K, seed=seed)
    X = wl.activation(T, K, seed=seed + 1)
    Y, A4, oq, oc, oh = run_fwd(qb, W, X, bits, G)
    r = np.random.default_rng(seed)
    ts = np.concatenate([r.integers(0, T, n_samples), [0, T - 1, 0, T - 1]])
    ns = np.concatenate([r.integers(0, N, n_samples), [0, N - 1, N - 1, 0]])
    Ys, A4s = oracle.qlinear_fwd_sampled(oq, CLIP, oc, oh, bits, ts, ns)
    assert (A4[ts, ns] == A4s).all()
    assert_rel(Y[ts, ns], Ys)
    # property that holds at any size: column sums of A4 against an exact integer identity
    # sum_t A4[t,n] = sum_j (2c'+1) * sum_t (2x'+1)
    colx = (2 * oq.astype(np.int64) + 1).sum(0)
    L = 2 ** bits - 1
    ref = ((2 * oc.astype(np.int64) - L) * colx[None, :]).sum(1)
    assert (A4.astype(np.int64).sum(0) == ref).all()


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("lin", wl.BERT_BASE_LINEARS, ids=[l[0] for l in wl.BERT_BASE_LINEARS])
def test_forward_config2_full_size(qb, bits, lin):
    """Configuration 2: the four linears of a BERT-base layer at T = 4096, every bit-width."""
    name, N, K = lin
    sampled_fwd_check(qb, 4096, N, K, 128, bits, seed=wl.config_seed(1, N + K + bits))


def test_forward_qkv_per_matrix_grouping(qb):
    """Fused QKV with 3 x 128 groups reproduces the paper's per-matrix grouping."""
    sampled_fwd_check(qb, 4096, 2304, 768, 384, 4, seed=wl.config_seed(1, 77))


@pytest.mark.parametrize("bits", (2, 3))
@pytest.mark.parametrize("lin", wl.BERT_LARGE_LINEARS, ids=[l[0] for l in wl.BERT_LARGE_LINEARS])
def test_forward_config5_bert_large(qb, bits, lin):
    """Configuration 5 shapes (T = 64 x 512) at 2 and 3 bits."""
    name, N, K = lin
    sampled_fwd_check(qb, 32768, N, K, 128, bits, seed=wl.config_seed(4, N + K + bits), n_samples=2048)


def test_forward_config4_mixed_bits(qb):
    """Configuration 4: T = 32 x 384, per-layer bits drawn by seed, plus the paper's Table 6/7 rows."""
    bits_list = wl.layer_bits(12, seed=wl.config_seed(3, 0))
    assert set(bits_list) <= set(BITS)
    for b in sorted(set(bits_list) | set(wl.PAPER_BITS_2_3["SST-2"]) | set(wl.PAPER_BITS_2_4["SST-2"])):
        sampled_fwd_check(qb, 12288, 768, 3072, 128, b, seed=wl.config_seed(3, b), n_samples=1024)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", [(4096, 768, 768), (4096, 2304, 768), (4096, 3072, 768), (4096, 768, 3072),
                                   (4096, 1024, 1024), (32768, 1024, 1024), (2048, 768, 192), (1000, 130, 256),
                                   (300, 96, 128), (129, 200, 384), (4096, 768, 192), (512, 768, 2048)])
def test_forward_plain_call_matches_checked_call(qb, bits, shape):
    """The call as bench.py makes it (no debug output: interior tiles take the straight-line streaming-store
    path) must give bit for bit the Y of the call with the debug output (every element checked), which the
    other tests compare with the oracle.  The shapes walk through every branch of the tile dispatch: 128x96
    tiles on three SIMDs, role-split 128x128, two plain workgroups per CU, the register-staged kernel with
    128x128 tiles for K not a multiple of 128 and with 32x64 tiles (64, 128 and 256 features per step) for
    problems of few tiles, ragged T and N, N not a multiple of 4; with and without bias."""
    T, N, K = shape
    G = 128 if N % 128 == 0 else (N // 2 if N % 2 == 0 else 1)
    say("fwd plain vs checked", shape, "bits", bits)
    W = wl.weight(N, K, seed=7 * N + K + bits).to(DEV)
    X = wl.activation(T, K, seed=T + 3 * K + bits).to(DEV)
    packed, h, m, rs_w = qb.qb_quantize_groupwise(W, bits, G)
    Xq, rs_x = qb.qb_quantize_act(X, CLIP)
    for bias in (None, wl.activation(1, N, seed=5)[0].contiguous().to(DEV)):
        Y_checked, A4 = qb.qb_qlinear_fwd(Xq, rs_x, CLIP, packed, h, rs_w, bits, G, N, bias=bias, want_a4=True)
        Y_plain = torch.full((T, N), float("nan"), dtype=torch.float32, device=DEV)
        qb.qb_qlinear_fwd(Xq, rs_x, CLIP, packed, h, rs_w, bits, G, N, bias=bias, Y=Y_plain)
        torch.cuda.synchronize()
        assert torch.equal(Y_plain, Y_checked)
    # and the integer against the oracle on sampled outputs
    r = np.random.default_rng(T + N + K)
    ts, ns = r.integers(0, T, 512), r.integers(0, N, 512)
    oc, oh, _, _ = oracle.quantize_groupwise(W.cpu().numpy(), bits, G)
    oq, _ = oracle.quantize_act(X.cpu().numpy(), CLIP)
    Ys, A4s = oracle.qlinear_fwd_sampled(oq, CLIP, oc, oh, bits, ts, ns)
    assert (A4.cpu().numpy()[ts, ns] == A4s).all()


# ---- backward ----------------------------------------------------------------------------------------
# ---- forward with 8-bit output --------------------------------------------------------------------------
def run_fwd_q8(qb, W, X, bits, G, clip_out, bias=None, act=0):
    N, K = W.shape
    packed, h, m, rs_w = qb.qb_quantize_groupwise(W.to(DEV), bits, G)
    Xq, rs_x = qb.qb_quantize_act(X.to(DEV), CLIP)
    Yq, rs_y = qb.qb_qlinear_fwd_q8(Xq, rs_x, CLIP, packed, h, rs_w, bits, G, N, clip_out,
                                    bias=None if bias is None else bias.to(DEV), act=act)
    torch.cuda.synchronize()
    oc, oh, _, _ = oracle.quantize_groupwise(W.numpy(), bits, G)
    oq, _ = oracle.quantize_act(X.numpy(), CLIP)
    return Yq.cpu().numpy(), rs_y.cpu().numpy(), oq, oc, oh


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", [(300, 384, 256, 128), (1000, 256, 384, 64), (517, 768, 768, 128), (70, 200, 128, 8),
                                   (1, 32, 128, 1), (2048, 1024, 128, 128)])
def test_forward_q8_output(qb, bits, shape):
    """Both tile layouts, ragged tails in T and N (N = 200: rows that are not a multiple of 16 bytes), with and
    without bias: codes and row sums equal the oracle's bit for bit."""
    T, N, K, G = shape
    say("fwd q8", shape, "bits", bits)
    W = wl.weight_uniform(N, K, seed=13 * N + K + bits, lo=-0.1, hi=0.1)
    X = wl.activation(T, K, seed=T + K + bits + 5)
    bias = (0.3 * wl.activation(1, N, seed=9)[0]).contiguous()
    for b, clip_out in ((None, 2.0), (bias, 0.75)):
        Yq, rs_y, oq, oc, oh = run_fwd_q8(qb, W, X, bits, G, clip_out, bias=b)
        yo, ro = oracle.qlinear_fwd_q8(oq, CLIP, oc, oh, bits, clip_out, bias=None if b is None else b.numpy(), openmp=True)
        assert (Yq == yo).all(), int((Yq != yo).sum())
        assert (rs_y == ro).all()
    assert Yq.min() == -128 and Yq.max() == 127 or T == 1


@pytest.mark.parametrize("bits", (3, 8))
def test_forward_q8_output_gelu(qb, bits):
    """GELU in front of the output quantizer: the binary32 erf may move a value across a rounding boundary, so
    codes may differ from the oracle's (binary64 erf) by one, rarely; row sums must fit the GPU's own codes."""
    T, N, K, G = 700, 768, 256, 128
    W = wl.weight_uniform(N, K, seed=77 + bits, lo=-0.1, hi=0.1)
    X = wl.activation(T, K, seed=78 + bits)
    bias = (0.3 * wl.activation(1, N, seed=9)[0]).contiguous()
    Yq, rs_y, oq, oc, oh = run_fwd_q8(qb, W, X, bits, G, 1.5, bias=bias, act=1)
    yo, ro = oracle.qlinear_fwd_q8(oq, CLIP, oc, oh, bits, 1.5, bias=bias.numpy(), act=1, openmp=True)
    d = np.abs(Yq.astype(np.int32) - yo.astype(np.int32))
    assert d.max() <= 1 and (d != 0).mean() < 1e-3, (int(d.max()), float((d != 0).mean()))
    assert (rs_y == Yq.astype(np.int64).sum(axis=1)).all()


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("lin", wl.BERT_BASE_LINEARS, ids=[l[0] for l in wl.BERT_BASE_LINEARS])
def test_forward_q8_config2_full_size(qb, bits, lin):
    """Configuration 2 shapes at T = 4096 as bench.py launches them (QKV also at 12288 tokens: nine tiles per
    workgroup): sampled token rows against the oracle (rows are independent), row sums of every row against the
    GPU's own codes."""
    name, N, K = lin
    T, G = (12288 if name == "qkv" and bits == 3 else 4096), 128
    say("fwd q8 full size", lin, "bits", bits)
    W = wl.weight(N, K, seed=wl.config_seed(1, N + K + bits))
    X = wl.activation(T, K, seed=wl.config_seed(1, N + K + bits) + 1)
    Yq, rs_y, oq, oc, oh = run_fwd_q8(qb, W, X, bits, G, 3.0)
    rows = np.concatenate([np.random.default_rng(N + K + bits).integers(0, T, 30), [0, T - 1]])
    yo, ro = oracle.qlinear_fwd_q8(oq[rows], CLIP, oc, oh, bits, 3.0, openmp=True)
    assert (Yq[rows] == yo).all()
    assert (rs_y[rows] == ro).all()
    assert (rs_y == Yq.astype(np.int64).sum(axis=1)).all()


# ---- dynamic (per-token) activation range ---------------------------------------------------------------------
@pytest.mark.parametrize("shape", [(1024, 768), (4096, 3072), (1, 64), (1023, 768), (7, 1024), (130, 4096), (33, 8192)])
def test_quantize_act_dynamic(qb, shape):
    T, K = shape
    say("act quant dynamic", shape)
    X = wl.activation(T, K, seed=T + K + 1)
    X[T // 2] *= 37.0
    if T > 4:
        X[3] = 0.0
    Xq, rs_x, hx = qb.qb_quantize_act_dyn(X.to(DEV))
    torch.cuda.synchronize()
    oq, ors, ohx = oracle.quantize_act_dyn(X.numpy())
    assert (Xq.cpu().numpy() == oq).all()
    assert (rs_x.cpu().numpy() == ors).all()
    assert (hx.cpu().numpy().view(np.uint32) == ohx.view(np.uint32)).all()


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", [(300, 384, 256, 128), (1000, 256, 192, 64), (517, 768, 768, 128), (70, 200, 128, 8),
                                   (2048, 1024, 128, 128), (2304, 1536, 128, 128), (4096, 768, 128, 128),
                                   (4096, 768, 192, 128)])
def test_forward_dynamic_scales(qb, bits, shape):
    """Per-token scales through every kernel that takes them (32x64 register-staged tiles, the 128x128 one for K not a
    multiple of 128, both role-split layouts), ragged T and N, with and without bias."""
    T, N, K, G = shape
    say("fwd dynamic", shape, "bits", bits)
    W = wl.weight_uniform(N, K, seed=17 * N + K + bits, lo=-0.1, hi=0.1)
    X = wl.activation(T, K, seed=T + K + bits + 9)
    X[T // 3] *= 11.0
    bias = (0.3 * wl.activation(1, N, seed=9)[0]).contiguous()
    packed, h, m, rs_w = qb.qb_quantize_groupwise(W.to(DEV), bits, G)
    Xq, rs_x, hx = qb.qb_quantize_act_dyn(X.to(DEV))
    oc, oh, _, _ = oracle.quantize_groupwise(W.numpy(), bits, G)
    oq, _, ohx = oracle.quantize_act_dyn(X.numpy())
    for b in (None, bias):
        Y, A4 = qb.qb_qlinear_fwd_dyn(Xq, rs_x, hx, packed, h, rs_w, bits, G, N, bias=None if b is None else b.to(DEV),
                                      want_a4=True)
        torch.cuda.synchronize()
        Yo, A4o = oracle.qlinear_fwd_dyn(oq, ohx, oc, oh, bits, bias=None if b is None else b.numpy(), openmp=True)
        assert (A4.cpu().numpy() == A4o).all()
        if b is None:
            assert_rel(Y.cpu().numpy(), Yo)
        else:
            assert np.abs(Y.cpu().numpy() - Yo).max() <= 1e-6 * max(np.abs(Yo).max(), np.abs(b.numpy()).max())
        Y2 = qb.qb_qlinear_fwd_dyn(Xq, rs_x, hx, packed, h, rs_w, bits, G, N, bias=None if b is None else b.to(DEV))
        torch.cuda.synchronize()
        assert torch.equal(Y2, Y)   # the call without the debug output


@pytest.mark.parametrize("shape", [(1, 64), (5, 192), (1000, 768), (4096, 3072), (257, 4096), (3, 16384)])
def test_quantize_act_dynamic_tensor(qb, shape):
    """One max-abs range for the whole tensor: codes, row sums, the range and the per-row scales bit for bit; a
    second call into the same buffers with a smaller tensor (the range must not survive from the first); zeros."""
    T, K = shape
    say("act quant dynamic, per tensor", shape)
    X = wl.activation(T, K, seed=T + K + 2)
    X[T // 2, K // 3] = 41.5          # the maximum, somewhere in the middle
    Xq, rs_x, hx, c = qb.qb_quantize_act_dyn_tensor(X.to(DEV))
    torch.cuda.synchronize()
    oq, ors, ohx = oracle.quantize_act_dyn_tensor(X.numpy())
    assert c.cpu().numpy()[0] == np.abs(X.numpy()).max()
    assert (Xq.cpu().numpy() == oq).all()
    assert (rs_x.cpu().numpy() == ors).all()
    assert (hx.cpu().numpy().view(np.uint32) == np.float32(ohx).view(np.uint32)).all()
    X2 = (0.01 * X).contiguous()
    qb.qb_quantize_act_dyn_tensor(X2.to(DEV), Xq, rs_x, hx, c)
    torch.cuda.synchronize()
    oq, ors, ohx = oracle.quantize_act_dyn_tensor(X2.numpy())
    assert (Xq.cpu().numpy() == oq).all() and (rs_x.cpu().numpy() == ors).all()
    assert (hx.cpu().numpy().view(np.uint32) == np.float32(ohx).view(np.uint32)).all()
    qb.qb_quantize_act_dyn_tensor(torch.zeros_like(X).to(DEV), Xq, rs_x, hx, c)
    torch.cuda.synchronize()
    assert (Xq == -128).all() and (rs_x == -128 * K).all() and (hx == 0).all() and (c == 0).all()


@pytest.mark.parametrize("bits", BITS)
def test_forward_dynamic_tensor_range_equals_fixed_clip(qb, bits):
    """Quantize with the tensor's own range, multiply with the per-token-scale forward: the oracle's result, and the
    fixed-clip forward's at clip = max|X| bit for bit."""
    T, N, K, G = 777, 768, 768, 128
    say("fwd dynamic, per tensor", (T, N, K), "bits", bits)
    W = wl.weight(N, K, seed=3 + bits)
    X = wl.activation(T, K, seed=5 + bits)
    packed, h, m, rs_w = qb.qb_quantize_groupwise(W.to(DEV), bits, G)
    Xq, rs_x, hx, c = qb.qb_quantize_act_dyn_tensor(X.to(DEV))
    Y, A4 = qb.qb_qlinear_fwd_dyn(Xq, rs_x, hx, packed, h, rs_w, bits, G, N, want_a4=True)
    Y1 = qb.qb_qlinear_fwd(Xq, rs_x, float(c.item()), packed, h, rs_w, bits, G, N)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y1)
    oc, oh, _, _ = oracle.quantize_groupwise(W.numpy(), bits, G)
    oq, _, ohx = oracle.quantize_act_dyn_tensor(X.numpy())
    Yo, A4o = oracle.qlinear_fwd_dyn(oq, np.full(T, ohx, np.float32), oc, oh, bits, openmp=True)
    assert (A4.cpu().numpy() == A4o).all()
    assert_rel(Y.cpu().numpy(), Yo)


def rel_fro(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b))


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", [(300, 160, 192, 8), (65, 6, 64, 6), (513, 768, 768, 128), (1000, 96, 320, 96),
                                   (4100, 1000, 1088, 8), (8192, 96, 64, 96)])
def test_backward_full_compare(qb, bits, shape):
    """Whole dX and dW against the oracle.  The last two shapes: 128 x 192 tiles with ragged edges in both directions and
    N not a multiple of 64; and one dW tile whose 128 contraction steps are shared by 32 workgroups (a long chain of
    partial sums)."""
    T, N, K, G = shape
    say("bwd full", shape, "bits", bits)
    W = wl.weight(N, K, seed=N + K + bits)
    X = wl.activation(T, K, seed=T + bits)
    dY = wl.grad_output_bf16(T, N, seed=T + N)
    packed, h, rs_w, oc, oh = check_quantize(qb, W, bits, G)
    Xq, rs_x = qb.qb_quantize_act(X.to(DEV), CLIP)
    dX, dW = qb.qb_qlinear_bwd_ste(dY.to(DEV), Xq, CLIP, packed, h, bits, G)
    torch.cuda.synchronize()
    oq, _ = oracle.quantize_act(X.numpy(), CLIP)
    odX, odW = oracle.qlinear_bwd_ste(wl.bf16_bits(dY), oq, CLIP, oc, oh, bits, openmp=True)
    assert rel_fro(dX.float().cpu().numpy(), odX) <= 2e-2
    assert rel_fro(dW.cpu().numpy(), odW) <= 2e-2
    # dW is accumulated in fp32 from exact bf16 products: much tighter than the bf16 bound
    assert rel_fro(dW.cpu().numpy(), odW) <= 1e-4
    # only one output requested: the workgroups then share the contraction steps differently, so the fp32 sums are
    # added in another (equally fixed) order and a result may land on the neighbouring bf16 value
    dX2, none = qb.qb_qlinear_bwd_ste(dY.to(DEV), Xq, CLIP, packed, h, bits, G, want_dw=False)
    assert none is None and rel_fro(dX2.float().cpu().numpy(), odX) <= 2e-2
    a, b = dX2.float().cpu().numpy(), dX.float().cpu().numpy()
    assert (np.abs(a - b) <= 2.0 ** -7 * np.abs(b) + 1e-5 * np.abs(b).max()).all()
    # the same call again gives the same bits
    dX3, _ = qb.qb_qlinear_bwd_ste(dY.to(DEV), Xq, CLIP, packed, h, bits, G, want_dw=False)
    assert torch.equal(dX3, dX2)


@pytest.mark.parametrize("bits", [3, 8])
@pytest.mark.parametrize("shape", [(300, 160, 192, 8), (65, 6, 64, 6), (1500, 768, 768, 128), (256, 3072, 768, 128),
                                   (1000, 96, 320, 96), (4100, 1000, 1088, 8), (8192, 96, 64, 96)])
def test_backward_clamp_masked(qb, bits, shape):
    """The backward that keeps the clamp's derivative: against the oracle (norms), exact zeros where the value lay
    outside its range, the plain backward's bits everywhere else, values at the range's ends pass; with tiles
    that one workgroup computes alone and tiles shared between workgroups, both tile shapes, and with one side masked
    only."""
    T, N, K, G = shape
    say("bwd masked", shape, "bits", bits)
    clip = 1.5
    W = wl.weight(N, K, seed=N + K + bits)
    X = wl.activation(T, K, seed=T + bits)
    X[0, 0], X[0, 1] = clip, -clip
    dY = wl.grad_output_bf16(T, N, seed=T + N)
    m_in = (0.5 * W.abs().reshape(G, -1).max(dim=1).values).contiguous()
    W[0, 0] = m_in[0]
    packed, h, rs_w = qb.qb_quantize_groupwise_clip(W.to(DEV), bits, m_in.to(DEV))
    Xq, rs_x = qb.qb_quantize_act(X.to(DEV), clip)
    dYd, Xd, Wd, md = dY.to(DEV), X.to(DEV), W.to(DEV), m_in.to(DEV)
    dX0, dW0 = qb.qb_qlinear_bwd_ste(dYd, Xq, clip, packed, h, bits, G)
    dX, dW = qb.qb_qlinear_bwd_ste_masked(dYd, Xq, clip, packed, h, bits, G, X=Xd, W=Wd, m=md)
    torch.cuda.synchronize()
    outX = X.abs() > clip
    outW = W.abs() > m_in.repeat_interleave(N // G)[:, None]
    assert outX.sum() > 0 and outW.sum() > 0 and not outX[0, 0] and not outX[0, 1] and not outW[0, 0]
    assert torch.equal(dX.cpu(), torch.where(outX, torch.zeros_like(dX0.cpu()), dX0.cpu()))
    assert torch.equal(dW.cpu(), torch.where(outW, torch.zeros_like(dW0.cpu()), dW0.cpu()))
    oc, oh, _ = oracle.quantize_groupwise_clip(W.numpy(), bits, m_in.numpy())
    oq, _ = oracle.quantize_act(X.numpy(), clip)
    odX, odW = oracle.qlinear_bwd_ste_masked(wl.bf16_bits(dY), oq, clip, oc, oh, bits, X=X.numpy(), W=W.numpy(),
                                             m=m_in.numpy(), openmp=True)
    assert ((odX == 0) == outX.numpy()).all() and ((odW == 0) == outW.numpy()).all()
    assert rel_fro(dX.float().cpu().numpy(), odX) <= 2e-2
    assert rel_fro(dW.cpu().numpy(), odW) <= 1e-4
    # one side only
    a, b = qb.qb_qlinear_bwd_ste_masked(dYd, Xq, clip, packed, h, bits, G, X=Xd)
    assert torch.equal(a, dX) and torch.equal(b, dW0)
    a, b = qb.qb_qlinear_bwd_ste_masked(dYd, Xq, clip, packed, h, bits, G, W=Wd, m=md)
    assert torch.equal(a, dX0) and torch.equal(b, dW)


def test_backward_clamp_masked_full_size_tall_tiles(qb):
    """FFN-down at T = 4096 (dX runs on 256 x 96 tiles): the masked result is the plain one with exact zeros where the
    activation lay outside its range; sampled entries against the oracle."""
    T, N, K, G, bits, clip = 4096, 768, 3072, 128, 3, 1.5
    say("bwd masked, tall tiles", (T, N, K))
    W = wl.weight(N, K, seed=5)
    X = wl.activation(T, K, seed=6)
    dY = wl.grad_output_bf16(T, N, seed=7)
    packed, h, m, rs_w = qb.qb_quantize_groupwise(W.to(DEV), bits, G)
    Xd = X.to(DEV)
    Xq, _ = qb.qb_quantize_act(Xd, clip)
    dX0, _ = qb.qb_qlinear_bwd_ste(dY.to(DEV), Xq, clip, packed, h, bits, G, want_dw=False)
    dX, _ = qb.qb_qlinear_bwd_ste_masked(dY.to(DEV), Xq, clip, packed, h, bits, G, X=Xd, want_dw=False)
    torch.cuda.synchronize()
    outX = X.abs() > clip
    assert torch.equal(dX.cpu(), torch.where(outX, torch.zeros_like(dX0.cpu()), dX0.cpu()))
    oc, oh, _, _ = oracle.quantize_groupwise(W.numpy(), bits, G)
    r = np.random.default_rng(11)
    ts, js = r.integers(0, T, 2048), r.integers(0, K, 2048)
    ref = oracle.bwd_dx_sampled(wl.bf16_bits(dY), oc, oh, bits, ts, js)
    got = dX0.float().cpu().numpy()[ts, js]
    assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= 2e-2


@pytest.mark.parametrize("lin", wl.BERT_BASE_LINEARS, ids=[l[0] for l in wl.BERT_BASE_LINEARS])
def test_backward_config3_full_size(qb, lin):
    """Configuration 3: T = 4096, 3-bit weights, 128 groups; sampled entries + norms."""
    name, N, K = lin
    T, bits, G = 4096, 3, 128
    say("bwd cfg3", lin)
    W = wl.weight(N, K, seed=wl.config_seed(2, N + K))
    X = wl.activation(T, K, seed=wl.config_seed(2, 1))
    dY = wl.grad_output_bf16(T, N, seed=wl.config_seed(2, 2))
    packed, h, rs_w, oc, oh = check_quantize(qb, W, bits, G)
    Xq, _ = qb.qb_quantize_act(X.to(DEV), CLIP)
    dX, dW = qb.qb_qlinear_bwd_ste(dY.to(DEV), Xq, CLIP, packed, h, bits, G)
    torch.cuda.synchronize()
    oq, _ = oracle.quantize_act(X.numpy(), CLIP)
    r = np.random.default_rng(N + K)
    n_s = 2048
    ts, js, ns = r.integers(0, T, n_s), r.integers(0, K, n_s), r.integers(0, N, n_s)
    bits16 = wl.bf16_bits(dY)
    sdx = oracle.bwd_dx_sampled(bits16, oc, oh, bits, ts, js)
    sdw = oracle.bwd_dw_sampled(bits16, oq, CLIP, ns, js)
    assert rel_fro(dX.float().cpu().numpy()[ts, js], sdx) <= 2e-2
    assert rel_fro(dW.cpu().numpy()[ns, js], sdw) <= 2e-2


# ---- embedding -------------------------------------------------------------------------------------------
@pytest.mark.parametrize("shape", [(30522, 1024, 128, 32768), (1000, 64, 8, 100), (517, 768, 128, 1), (300, 128, 1, 50),
                                   (64, 192, 192, 10), (203, 2304, 36, 20), (100, 192, 64, 5)])
def test_embedding(qb, shape):
    V, d, G, n = shape
    say("embedding", shape)
    E = wl.embedding_table(V, d, seed=wl.config_seed(4, V + d))
    ids = wl.token_ids(n, V, seed=wl.config_seed(4, 1))
    codes, h, m = qb.qb_embedding_quantize(E.to(DEV), G)
    out = qb.qb_embedding_gather(codes, h, G, ids.to(DEV))
    torch.cuda.synchronize()
    oc, oh, om = oracle.embedding_quantize(E.numpy(), G)
    assert (codes.cpu().numpy() == oc).all()
    assert (h.cpu().numpy().view(np.uint32) == oh.view(np.uint32)).all()
    assert (m.cpu().numpy().view(np.uint32) == om.view(np.uint32)).all()
    oo = oracle.embedding_gather(oc, oh, ids.numpy())
    assert_rel(out.cpu().numpy(), oo.astype(np.float32), tol=1e-6)
    # empty lookup
    empty = qb.qb_embedding_gather(codes, h, G, ids[:0].to(DEV))
    assert empty.shape == (0, d)
    # an id outside the table yields a zero row instead of reading out of bounds
    bad = torch.tensor([V, -1, 0], dtype=torch.int64)
    ob = qb.qb_embedding_gather(codes, h, G, bad.to(DEV)).cpu()
    assert (ob[:2] == 0).all() and (ob[2].numpy() == oracle.embedding_gather(oc, oh, np.array([0]))[0].astype(np.float32)).all()


@pytest.mark.parametrize("shape", [(30522, 768, 128, 4096), (1000, 64, 8, 100), (517, 768, 128, 1), (300, 128, 1, 50),
                                   (64, 192, 192, 10), (203, 2304, 36, 20), (100, 192, 64, 5)])
def test_embedding_4bit(qb, shape):
    """4-bit table (the paper's mixed-precision embedding): packed bytes equal the oracle's codes packed as a
    little-endian bit stream, scales bit for bit, the gather within 1e-6; the 8-bit call through the same entry
    point equals the dedicated one."""
    V, d, G, n = shape
    say("embedding 4-bit", shape)
    E = wl.embedding_table(V, d, seed=wl.config_seed(4, V + d + 4))
    ids = wl.token_ids(n, V, seed=wl.config_seed(4, 2))
    codes, h, m = qb.qb_embedding_quantize_bits(E.to(DEV), 4, G)
    out = qb.qb_embedding_gather_bits(codes, h, 4, G, ids.to(DEV))
    torch.cuda.synchronize()
    oc, oh, om = oracle.embedding_quantize(E.numpy(), G, bits=4)
    assert codes.shape == (V, d // 2)
    assert (codes.cpu().numpy() == oracle.pack(oc, 4)).all()
    assert (h.cpu().numpy().view(np.uint32) == oh.view(np.uint32)).all()
    assert (m.cpu().numpy().view(np.uint32) == om.view(np.uint32)).all()
    oo = oracle.embedding_gather(oc, oh, ids.numpy(), bits=4)
    assert_rel(out.cpu().numpy(), oo.astype(np.float32), tol=1e-6)
    bad = torch.tensor([V, -1, 0], dtype=torch.int64)
    ob = qb.qb_embedding_gather_bits(codes, h, 4, G, bad.to(DEV)).cpu()
    assert (ob[:2] == 0).all() and (ob[2].numpy() == oracle.embedding_gather(oc, oh, np.array([0]), bits=4)[0].astype(np.float32)).all()
    c8, h8, m8 = qb.qb_embedding_quantize_bits(E.to(DEV), 8, G)
    c8b, h8b, m8b = qb.qb_embedding_quantize(E.to(DEV), G)
    assert torch.equal(c8, c8b) and torch.equal(h8, h8b) and torch.equal(m8, m8b)


def test_runs_are_deterministic(qb):
    """Integer accumulation is order independent and dW partial sums are added in a fixed order."""
    T, N, K, G, bits = 2048, 768, 768, 128, 3
    W = wl.weight(N, K, seed=1).to(DEV)
    X = wl.activation(T, K, seed=2).to(DEV)
    dY = wl.grad_output_bf16(T, N, seed=3).to(DEV)
    outs = []
    for _ in range(3):
        packed, h, m, rs_w = qb.qb_quantize_groupwise(W, bits, G)
        Xq, rs_x = qb.qb_quantize_act(X, CLIP)
        Y = qb.qb_qlinear_fwd(Xq, rs_x, CLIP, packed, h, rs_w, bits, G, N)
        dX, dW = qb.qb_qlinear_bwd_ste(dY, Xq, CLIP, packed, h, bits, G)
        torch.cuda.synchronize()
        outs.append((packed.clone(), Y.clone(), dX.clone(), dW.clone()))
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            assert torch.equal(a, b)


# ---- asymmetric group ranges --------------------------------------------------------------------------------------------
def shifted_weight(N, K, G, seed):
    """Groups with their own offsets: one-sided, shifted and near-symmetric ones, one constant group."""
    W = wl.weight(N, K, seed=seed)
    rows = N // G
    for g in range(G):
        blk = W[g * rows:(g + 1) * rows]
        if g % 4 == 0:
            blk.abs_()                       # one-sided
        elif g % 4 == 1:
            blk += 0.07 * (g % 5 + 1)        # shifted
        elif g % 4 == 2 and g > 2:
            blk.fill_(0.03125)               # constant
    return W.contiguous()


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", [(768, 768, 128), (2304, 768, 12), (768, 3072, 128), (6, 64, 6), (40, 192, 8), (1030, 64, 1),
                                   (4096, 1024, 2)])
def test_quantize_asymmetric_ranges(qb, bits, shape):
    """Codes, Delta and q0 (bit patterns) and row sums against the oracle; groups in one panel and groups split over
    panels and slices; a second call into the same buffers."""
    N, K, G = shape
    say("quantize asym", shape, "bits", bits)
    W = shifted_weight(N, K, G, seed=N + K + bits)
    packed, delta, q0, rs = qb.qb_quantize_groupwise_asym(W.to(DEV), bits, G)
    codes = qb.qb_unpack_codes(packed, N, K, bits)
    torch.cuda.synchronize()
    oc, od, oq0, ors = oracle.quantize_groupwise_asym(W.numpy(), bits, G)
    assert (delta.cpu().numpy().view(np.uint32) == od.view(np.uint32)).all()
    assert (q0.cpu().numpy() == oq0).all()
    assert (codes.cpu().numpy() == oc).all()
    assert (rs.cpu().numpy() == ors).all()
    W2 = (-0.5 * W).contiguous()
    qb.qb_quantize_groupwise_asym(W2.to(DEV), bits, G, packed, delta, q0, rs)
    codes = qb.qb_unpack_codes(packed, N, K, bits)
    torch.cuda.synchronize()
    oc, od, oq0, ors = oracle.quantize_groupwise_asym(W2.numpy(), bits, G)
    assert (delta.cpu().numpy().view(np.uint32) == od.view(np.uint32)).all() and (q0.cpu().numpy() == oq0).all()
    assert (codes.cpu().numpy() == oc).all() and (rs.cpu().numpy() == ors).all()


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", [(300, 160, 192, 8), (1, 32, 64, 1), (129, 130, 320, 10), (513, 768, 768, 128), (64, 6, 128, 6),
                                   (2048, 1024, 128, 128), (2304, 1536, 128, 128), (4096, 768, 256, 128), (100, 96, 2048, 96)])
def test_forward_asymmetric_ranges(qb, bits, shape):
    """Y against the oracle within 1e-6 of h_x*(Delta*|S| + |q0|*|R|) (the two products that are added), A4 bit for
    bit; through the register-staged kernel (few tiles, K not a multiple of 128) and both role-split layouts; ragged
    T and N; with bias."""
    T, N, K, G = shape
    say("fwd asym", shape, "bits", bits)
    W = shifted_weight(N, K, G, seed=3 * N + K + bits)
    X = wl.activation(T, K, seed=T + K + bits)
    bias = (0.3 * wl.activation(1, N, seed=11)[0]).contiguous()
    packed, delta, q0, rs_w = qb.qb_quantize_groupwise_asym(W.to(DEV), bits, G)
    Xq, rs_x = qb.qb_quantize_act(X.to(DEV), CLIP)
    oc, od, oq0, _ = oracle.quantize_groupwise_asym(W.numpy(), bits, G)
    oq, ors_x = oracle.quantize_act(X.numpy(), CLIP)
    Yo, S = oracle.qlinear_fwd_asym(oq, CLIP, oc, od, oq0, want_s=True, openmp=True)
    L = 2 ** bits - 1
    R = (2 * ors_x.astype(np.int64) + K)[:, None]
    rows = N // G
    dn = np.repeat(od.astype(np.float64), rows)[None, :]
    zn = np.repeat(oq0.astype(np.float64), rows)[None, :]
    bound = 1e-6 * (CLIP / 255.0) * (dn * np.abs(S) + np.abs(zn) * np.abs(R))
    for b in (None, bias):
        Y, A4 = qb.qb_qlinear_fwd_asym(Xq, rs_x, CLIP, packed, delta, q0, rs_w, bits, G, N,
                                       bias=None if b is None else b.to(DEV), want_a4=True)
        torch.cuda.synchronize()
        assert (A4.cpu().numpy().astype(np.int64) == 2 * S - L * R).all()
        ref = Yo.astype(np.float64) if b is None else oracle.qlinear_fwd_asym(oq, CLIP, oc, od, oq0, bias=b.numpy(), openmp=True)
        extra = 0 if b is None else 1e-6 * np.abs(b.numpy())[None, :]
        assert (np.abs(Y.cpu().numpy().astype(np.float64) - ref) <= bound + extra + 1e-30).all()
        Y2 = qb.qb_qlinear_fwd_asym(Xq, rs_x, CLIP, packed, delta, q0, rs_w, bits, G, N, bias=None if b is None else b.to(DEV))
        torch.cuda.synchronize()
        assert torch.equal(Y2, Y)


@pytest.mark.parametrize("shape", [(96, 64, 32768, 32), (2048, 768, 32768, 128)])
@pytest.mark.parametrize("bits", (2, 8))
def test_forward_asymmetric_maximum_K_and_extreme_codes(qb, bits, shape):
    """The longest contraction with operands at the ends of their ranges: S = sum (2x'+1) u reaches 255 * L * K
    (2.13e9 at 8 bits) and must stay inside int32 on the way (S = A4/2 + L*(R/2)); the register-staged and the
    role-split kernel."""
    T, N, K, G = shape
    say("fwd asym max K", shape, "bits", bits)
    L = 2 ** bits - 1
    W = torch.full((N, K), 0.1)
    W[:, ::2] = 0.3                     # every group holds its minimum and its maximum: codes 0 and L
    W[1::2] = 0.3                       # rows of all-L codes
    W[5, ::3] = 0.17
    X = torch.full((T, K), 6.0)         # x' = 127: 2x'+1 = 255
    X[1::3] = -6.0
    X[2::3] = wl.activation(T, K, seed=5)[2::3]
    packed, delta, q0, rs_w = qb.qb_quantize_groupwise_asym(W.to(DEV), bits, G)
    Xq, rs_x = qb.qb_quantize_act(X.to(DEV), CLIP)
    Y = qb.qb_qlinear_fwd_asym(Xq, rs_x, CLIP, packed, delta, q0, rs_w, bits, G, N)
    torch.cuda.synchronize()
    oc, od, oq0, _ = oracle.quantize_groupwise_asym(W.numpy(), bits, G)
    oq, ors_x = oracle.quantize_act(X.numpy(), CLIP)
    assert (qb.qb_unpack_codes(packed, N, K, bits).cpu().numpy() == oc).all()
    ts = np.arange(0, T, max(1, T // 48))
    Yo, S = oracle.qlinear_fwd_asym(oq[ts], CLIP, oc, od, oq0, want_s=True, openmp=True)
    assert int(np.abs(S).max()) == 255 * L * K
    R = (2 * ors_x[ts].astype(np.int64) + K)[:, None]
    rows = N // G
    dn = np.repeat(od.astype(np.float64), rows)[None, :]
    zn = np.repeat(oq0.astype(np.float64), rows)[None, :]
    bound = 1e-6 * (CLIP / 255.0) * (dn * np.abs(S) + np.abs(zn) * np.abs(R))
    assert (np.abs(Y.cpu().numpy()[ts].astype(np.float64) - Yo) <= bound).all()


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("shape", [(300, 160, 192, 8), (513, 768, 768, 128), (1000, 96, 320, 96)])
def test_backward_asymmetric_ranges(qb, bits, shape):
    T, N, K, G = shape
    say("bwd asym", shape, "bits", bits)
    W = shifted_weight(N, K, G, seed=N + K + bits)
    X = wl.activation(T, K, seed=T + bits)
    dY = wl.grad_output_bf16(T, N, seed=T + N)
    packed, delta, q0, rs_w = qb.qb_quantize_groupwise_asym(W.to(DEV), bits, G)
    Xq, rs_x = qb.qb_quantize_act(X.to(DEV), CLIP)
    dX, dW = qb.qb_qlinear_bwd_ste_asym(dY.to(DEV), Xq, CLIP, packed, delta, q0, bits, G)
    torch.cuda.synchronize()
    oc, od, oq0, _ = oracle.quantize_groupwise_asym(W.numpy(), bits, G)
    oq, _ = oracle.quantize_act(X.numpy(), CLIP)
    odX = oracle.qlinear_bwd_dx_asym(wl.bf16_bits(dY), oc, od, oq0, openmp=True)
    _, odW = oracle.qlinear_bwd_ste(wl.bf16_bits(dY), oq, CLIP, oc, np.ones(G, np.float32), bits, want_dx=False, openmp=True)
    assert rel_fro(dX.float().cpu().numpy(), odX) <= 2e-2
    assert rel_fro(dW.cpu().numpy(), odW) <= 1e-4


# ---- Hessian sensitivity: power iteration on the device ----------------------------------------------------------------
@pytest.mark.parametrize("case", ["dense-512", "diag-3000001", "zero"])
def test_power_iteration(qb, case):
    """Alg. 1 around a Hessian-vector product supplied as a callback, against the oracle's binary64 iteration from
    the same start vector: every step's estimate, and the final vector up to rounding.  A dense symmetric matrix with
    a known spectrum (top eigenvalue negative), a long diagonal operator (several partial sums per reduction, ragged
    tail), and the zero operator."""
    say("power iteration", case)
    r = np.random.default_rng(7)
    if case == "dense-512":
        n, iters = 512, 40
        Q, _ = np.linalg.qr(r.standard_normal((n, n)))
        spec = np.concatenate([[-5.0, 3.0], r.uniform(-2.0, 2.0, n - 2)])
        H = (Q * spec) @ Q.T
        H = (0.5 * (H + H.T)).astype(np.float32)
        Hd = torch.from_numpy(H).to(DEV)
        hv_gpu = lambda v, out: torch.mv(Hd, v, out=out)
        hv_cpu = lambda x: H.astype(np.float64) @ x
    elif case == "zero":
        n, iters = 1000, 3
        hv_gpu = lambda v, out: out.zero_()
        hv_cpu = lambda x: 0.0 * x
    else:
        n, iters = 3000001, 25
        d = r.uniform(-1.0, 1.0, n).astype(np.float32)
        d[12345], d[n - 1] = 4.0, -3.0
        dd = torch.from_numpy(d).to(DEV)
        hv_gpu = lambda v, out: torch.mul(dd, v, out=out)
        hv_cpu = lambda x: d.astype(np.float64) * x
    v0 = r.standard_normal(n).astype(np.float32)
    est, v = qb.qb_power_iteration(hv_gpu, torch.from_numpy(v0).to(DEV), iters)
    torch.cuda.synchronize()
    lam, vo = oracle.power_iteration(hv_cpu, v0, iters)
    est = est.cpu().numpy().astype(np.float64)
    if case == "zero":
        assert (est == 0).all() and (v == 0).all()
        return
    assert np.abs(est - lam).max() <= 1e-4 * np.abs(lam).max()
    vv = v.cpu().numpy().astype(np.float64)
    assert abs(np.linalg.norm(vv) - 1.0) < 1e-5
    assert np.abs(vv - vo).max() <= 2e-4
    top = -5.0 if case == "dense-512" else 4.0
    assert abs(est[-1] - top) < 1e-3 * abs(top) + (0.05 if case != "dense-512" else 0)


def test_power_iteration_callback_failure_is_reported(qb):
    """A product that fails ends the call: the exception of a Python callback comes back to the caller."""
    v = torch.ones(1000, dtype=torch.float32, device=DEV)

    def bad(v_, out_):
        raise ValueError("no product today")
    with pytest.raises(ValueError):
        qb.qb_power_iteration(bad, v, 3)
    torch.cuda.synchronize()


def test_mfma_probe_runs_and_leaves_its_sink_alone(qb):
    """The measurement aid: it launches, finishes and reports the operation count its kernel performs."""
    sink = torch.full((1,), 77, dtype=torch.int32, device=DEV)
    ops = qb.qb_probe_mfma_i8(8, 10, sink)
    torch.cuda.synchronize()
    assert ops == 8 * 4 * 10 * 4 * 65536 and int(sink.item()) == 77

