"""GPU parity at full size: whole-output comparisons of the kernels the benchmark times, the batched forward,
configuration 4 (12-layer stack at 32 x 384 tokens with per-layer bits) forward and backward, and per-element
bounds for the STE backward at configuration-3 size.  Everything goes through the C ABI; the reference is the
CPU oracle (its OpenMP build, the same source)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1909_05840_amd import workloads as wl

pytestmark = pytest.mark.gpu
BITS = (2, 3, 4, 8)
CLIP = 6.0
DEV = "cuda:0"
G = 128


def say(*a):
    print(*a, flush=True)


def quantized_inputs(qb, N, K, T, bits, seed, groups=G, uniform=False):
    W = wl.weight_uniform(N, K, seed=seed, lo=-0.1, hi=0.1) if uniform else wl.weight(N, K, seed=seed)
    X = wl.activation(T, K, seed=seed + 1)
    packed, h, m, rs_w = qb.qb_quantize_groupwise(W.to(DEV), bits, groups)
    Xq, rs_x = qb.qb_quantize_act(X.to(DEV), CLIP)
    oc, oh, _, ors = oracle.quantize_groupwise(W.numpy(), bits, groups)
    oq, orx = oracle.quantize_act(X.numpy(), CLIP)
    torch.cuda.synchronize()
    assert (qb.qb_unpack_codes(packed, N, K, bits).cpu().numpy() == oc).all()
    assert (Xq.cpu().numpy() == oq).all()
    assert (rs_w.cpu().numpy() == ors).all() and (rs_x.cpu().numpy() == orx).all()
    return dict(W=W, X=X, packed=packed, h=h, rs_w=rs_w, Xq=Xq, rs_x=rs_x, oc=oc, oh=oh, oq=oq)


def assert_rel(Y, Yo, tol=1e-6):
    err = np.abs(Y.astype(np.float64) - Yo)
    bad = err > tol * np.abs(Yo)
    assert not bad.any(), "%d elements outside %g relative, worst %g" % (bad.sum(), tol, (err / np.maximum(np.abs(Yo), 1e-300)).max())


# (T, N, K): every kernel the tile dispatch can choose for a large problem, at the benchmark's own sizes and with
# ragged edges: 128x96 tiles on three SIMDs (N = 768 at 4096 tokens; 4000 x 760 ragged in both directions),
# role-split 128x128 (4096 x 1024 x 1024; 2049 x 1530 ragged), two plain workgroups per CU (4096 x 3072 x 768;
# 4090 x 3000 ragged).
TIMED_KERNEL_SHAPES = [(4096, 768, 3072), (4096, 768, 768), (4096, 2304, 768), (4000, 760, 256), (4096, 1024, 1024),
                       (2049, 1530, 256), (4096, 3072, 768), (4090, 3000, 256)]


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", TIMED_KERNEL_SHAPES)
def test_forward_whole_output_of_timed_kernels(qb, bits, shape):
    """Y of the plain call (the launch bench.py times: streaming-store write-out) and A4 of the checked call, every
    element against the oracle."""
    T, N, K = shape
    groups = G if N % G == 0 else (N // 2 if N % 2 == 0 else 1)
    say("fwd whole output", shape, "bits", bits)
    d = quantized_inputs(qb, N, K, T, bits, seed=31 * N + K + bits, groups=groups)
    bias = wl.activation(1, N, seed=9)[0].contiguous()
    Y = torch.full((T, N), float("nan"), dtype=torch.float32, device=DEV)
    qb.qb_qlinear_fwd(d["Xq"], d["rs_x"], CLIP, d["packed"], d["h"], d["rs_w"], bits, groups, N, Y=Y)
    Yb = torch.full((T, N), float("nan"), dtype=torch.float32, device=DEV)
    qb.qb_qlinear_fwd(d["Xq"], d["rs_x"], CLIP, d["packed"], d["h"], d["rs_w"], bits, groups, N, bias=bias.to(DEV), Y=Yb)
    _, A4 = qb.qb_qlinear_fwd(d["Xq"], d["rs_x"], CLIP, d["packed"], d["h"], d["rs_w"], bits, groups, N, want_a4=True)
    torch.cuda.synchronize()
    Yo, A4o, _ = oracle.qlinear_fwd(d["oq"], CLIP, d["oc"], d["oh"], bits, openmp=True)
    assert (A4.cpu().numpy() == A4o).all()
    Yh = Y.cpu().numpy()
    assert_rel(Yh, Yo)
    assert (Yh[A4o == 0] == 0).all()
    # with bias: (Y + b) - b recovers Y to a rounding of the sum
    Ybh = Yb.cpu().numpy().astype(np.float64)
    b = bias.numpy().astype(np.float64)[None, :]
    assert (np.abs(Ybh - (Yo + b)) <= 1e-6 * np.abs(Yo) + 2.0 ** -23 * np.abs(Yo + b)).all()


def test_forward_batched_matches_single_calls(qb):
    """The benchmark's 16 jobs (4 linears x 4 bit-widths at 4096 tokens) plus jobs that do not share launches (few
    tiles, K not a multiple of 128, N not a multiple of 96, a very large one) in one call: every Y bit for bit the Y
    of the single call, and one job of every bit-width element by element against the oracle."""
    jobs, singles, checks = [], [], []
    shapes = [(4096, N, K) for (_, N, K) in wl.BERT_BASE_LINEARS]
    extra = [(128, 768, 3072, 4), (1000, 130, 192, 3), (2049, 1530, 256, 2), (4096, 1024, 1024, 8), (300, 96, 128, 4),
             (16384, 1024, 1024, 2), (4096, 768, 768, 4)]
    case = 0
    for bits in BITS:
        for (T, N, K) in shapes:
            d = quantized_inputs(qb, N, K, T, bits, seed=17 * N + K + bits + case)
            bias = wl.activation(1, N, seed=case)[0].contiguous().to(DEV) if case % 3 == 0 else None
            jobs.append(dict(Xq=d["Xq"], rs_x=d["rs_x"], clip=CLIP, packed=d["packed"], h=d["h"], rs_w=d["rs_w"], bits=bits,
                             groups=G, N=N, bias=bias))
            singles.append(qb.qb_qlinear_fwd(d["Xq"], d["rs_x"], CLIP, d["packed"], d["h"], d["rs_w"], bits, G, N, bias=bias))
            if (N, K) == (768, 3072):
                checks.append((len(jobs) - 1, d, bits, bias))
            case += 1
    for (T, N, K, bits) in extra:
        groups = G if N % G == 0 else (N // 2 if N % 2 == 0 else 1)
        d = quantized_inputs(qb, N, K, T, bits, seed=5 * N + K + T, groups=groups)
        jobs.append(dict(Xq=d["Xq"], rs_x=d["rs_x"], clip=CLIP, packed=d["packed"], h=d["h"], rs_w=d["rs_w"], bits=bits,
                         groups=groups, N=N, bias=None))
        singles.append(qb.qb_qlinear_fwd(d["Xq"], d["rs_x"], CLIP, d["packed"], d["h"], d["rs_w"], bits, groups, N))
    for j in jobs:  # outputs pre-filled: every element must be written by the batched call
        T = j["Xq"].shape[0]
        j["Y"] = torch.full((T, j["N"]), float("nan"), dtype=torch.float32, device=DEV)
    say("fwd batched", len(jobs), "jobs")
    Ys = qb.qb_qlinear_fwd_batched(jobs)
    torch.cuda.synchronize()
    for i, (Yb, Y1) in enumerate(zip(Ys, singles)):
        assert torch.equal(Yb, Y1), "job %d differs from the single call" % i
    for (i, d, bits, bias) in checks:
        Yo, _, _ = oracle.qlinear_fwd(d["oq"], CLIP, d["oc"], d["oh"], bits, openmp=True)
        Yh = Ys[i].cpu().numpy().astype(np.float64)
        if bias is not None:
            b = bias.cpu().numpy().astype(np.float64)[None, :]
            assert (np.abs(Yh - (Yo + b)) <= 1e-6 * np.abs(Yo) + 2.0 ** -23 * np.abs(Yo + b)).all()
        else:
            assert_rel(Yh, Yo)
    # an empty list is a valid call
    assert qb.qb_qlinear_fwd_batched([]) == []


def test_forward_batched_rejects_bad_jobs_before_launching(qb):
    d = quantized_inputs(qb, 768, 768, 256, 4, seed=3)
    good = dict(Xq=d["Xq"], rs_x=d["rs_x"], clip=CLIP, packed=d["packed"], h=d["h"], rs_w=d["rs_w"], bits=4, groups=G, N=768)
    Y0 = torch.full((256, 768), 7.0, dtype=torch.float32, device=DEV)
    bad = dict(good, bits=5)
    with pytest.raises(qb.QBError) as e:
        qb.qb_qlinear_fwd_batched([dict(good, Y=Y0), bad])
    assert e.value.status == 2
    torch.cuda.synchronize()
    assert (Y0 == 7.0).all()  # nothing was launched


# ---- configuration 4: 12-layer stack, T = 32 x 384 = 12288, per-layer bits ---------------------------------------
CFG4_T = 12288


def cfg4_bit_vectors():
    vecs = {"seeded": wl.layer_bits(12, seed=wl.config_seed(3, 0)), "table6-SST-2": wl.PAPER_BITS_2_3["SST-2"],
            "table7-SST-2": wl.PAPER_BITS_2_4["SST-2"]}
    return vecs


def sampled_forward(qb, T, N, K, bits, seed, n_samples=1024):
    d = quantized_inputs(qb, N, K, T, bits, seed=seed)
    Y, A4 = qb.qb_qlinear_fwd(d["Xq"], d["rs_x"], CLIP, d["packed"], d["h"], d["rs_w"], bits, G, N, want_a4=True)
    Yp = torch.full((T, N), float("nan"), dtype=torch.float32, device=DEV)
    qb.qb_qlinear_fwd(d["Xq"], d["rs_x"], CLIP, d["packed"], d["h"], d["rs_w"], bits, G, N, Y=Yp)
    torch.cuda.synchronize()
    assert torch.equal(Y, Yp)
    Y, A4 = Y.cpu().numpy(), A4.cpu().numpy()
    r = np.random.default_rng(seed)
    ts = np.concatenate([r.integers(0, T, n_samples), [0, T - 1, 0, T - 1]])
    ns = np.concatenate([r.integers(0, N, n_samples), [0, N - 1, N - 1, 0]])
    Ys, A4s = oracle.qlinear_fwd_sampled(d["oq"], CLIP, d["oc"], d["oh"], bits, ts, ns)
    assert (A4[ts, ns] == A4s).all()
    assert_rel(Y[ts, ns], Ys)
    # exact at any size: column sums and row sums of A4 against integer identities
    L = 2 ** bits - 1
    colx = (2 * d["oq"].astype(np.int64) + 1).sum(0)
    assert (A4.astype(np.int64).sum(0) == ((2 * d["oc"].astype(np.int64) - L) * colx[None, :]).sum(1)).all()
    roww = (2 * d["oc"].astype(np.int64) - L).sum(0)
    assert (A4.astype(np.int64).sum(1) == ((2 * d["oq"].astype(np.int64) + 1) * roww[None, :]).sum(1)).all()
    return d


@pytest.mark.parametrize("lin", wl.BERT_BASE_LINEARS, ids=[l[0] for l in wl.BERT_BASE_LINEARS])
def test_config4_forward_all_linears(qb, lin):
    """Every linear of the layer at 12288 tokens, at every bit-width the seeded vector and the paper's Table 6 / 7
    rows assign to some layer: sampled outputs, and the exact column- and row-sum identities over the whole A4."""
    name, N, K = lin
    widths = sorted(set(b for v in cfg4_bit_vectors().values() for b in v))
    assert set(widths) <= set(BITS)
    for bits in widths:
        say("cfg4 fwd", lin, "bits", bits)
        sampled_forward(qb, CFG4_T, N, K, bits, seed=wl.config_seed(3, N + K + bits))


@pytest.mark.parametrize("lin", wl.BERT_BASE_LINEARS, ids=[l[0] for l in wl.BERT_BASE_LINEARS])
def test_config4_backward_all_linears(qb, lin):
    """STE backward at 12288 tokens with the bit-widths of the seeded per-layer vector: sampled entries of dX and dW
    against the oracle (relative Frobenius over the sample, and a bound per sampled element)."""
    name, N, K = lin
    T = CFG4_T
    for bits in sorted(set(cfg4_bit_vectors()["seeded"])):
        say("cfg4 bwd", lin, "bits", bits)
        d = quantized_inputs(qb, N, K, T, bits, seed=wl.config_seed(3, 100 + N + K + bits))
        dY = wl.grad_output_bf16(T, N, seed=wl.config_seed(3, 200 + N + bits))
        dX, dW = qb.qb_qlinear_bwd_ste(dY.to(DEV), d["Xq"], CLIP, d["packed"], d["h"], bits, G)
        torch.cuda.synchronize()
        r = np.random.default_rng(N + K + bits)
        n_s = 4096
        ts, js, ns = r.integers(0, T, n_s), r.integers(0, K, n_s), r.integers(0, N, n_s)
        b16 = wl.bf16_bits(dY)
        sdx = oracle.bwd_dx_sampled(b16, d["oc"], d["oh"], bits, ts, js)
        sdw = oracle.bwd_dw_sampled(b16, d["oq"], CLIP, ns, js)
        gdx = dX.float().cpu().numpy()[ts, js].astype(np.float64)
        gdw = dW.cpu().numpy()[ns, js].astype(np.float64)
        assert np.linalg.norm(gdx - sdx) / np.linalg.norm(sdx) <= 2e-2
        assert np.linalg.norm(gdw - sdw) / np.linalg.norm(sdw) <= 1e-4
        # per element: magnitude sums of the products bound the rounding of operands and accumulation
        dYf = dY.float().numpy().astype(np.float64)
        What = oracle.dequantize_groupwise(d["oc"], d["oh"], bits).astype(np.float64)
        sabs_x = np.einsum("sn,ns->s", np.abs(dYf[ts, :]), np.abs(What[:, js]))
        assert (np.abs(gdx - sdx) <= 2.0 ** -8 * np.abs(sdx) + 2.0 ** -8 * sabs_x).all()
        Xhat = oracle.dequantize_act(d["oq"], CLIP).astype(np.float64)
        sabs_w = np.einsum("ts,ts->s", np.abs(dYf[:, ns]), np.abs(Xhat[:, js]))
        assert (np.abs(gdw - sdw) <= 2.0 ** -10 * sabs_w).all()


# ---- configuration 3 at full size: whole matrices ------------------------------------------------------------------
@pytest.mark.parametrize("lin", wl.BERT_BASE_LINEARS, ids=[l[0] for l in wl.BERT_BASE_LINEARS])
def test_backward_config3_whole_matrices(qb, lin):
    """T = 4096, 3-bit weights: dX and dW complete against the oracle's binary64 products: relative Frobenius norm
    over the whole matrix and a bound for every element.  Error model: What is rounded to bf16 (2^-9 relative per
    operand element), products are accumulated in fp32 (at most N * 2^-24 of the magnitude sum), dX is rounded to
    bf16 on the way out (2^-9 of its value); dW has exact operands (dY and 2x'+1 are bf16 values) and differs by
    the fp32 summation order only (at most T * 2^-24 of the magnitude sum)."""
    name, N, K = lin
    T, bits = 4096, 3
    say("bwd cfg3 whole", lin)
    d = quantized_inputs(qb, N, K, T, bits, seed=wl.config_seed(2, N + K))
    dY = wl.grad_output_bf16(T, N, seed=wl.config_seed(2, 2))
    dX, dW = qb.qb_qlinear_bwd_ste(dY.to(DEV), d["Xq"], CLIP, d["packed"], d["h"], bits, G)
    torch.cuda.synchronize()
    odX, odW = oracle.qlinear_bwd_ste(wl.bf16_bits(dY), d["oq"], CLIP, d["oc"], d["oh"], bits, openmp=True)
    gdx = dX.float().cpu().numpy().astype(np.float64)
    gdw = dW.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(gdx - odX) / np.linalg.norm(odX) <= 2e-2
    assert np.linalg.norm(gdw - odW) / np.linalg.norm(odW) <= 1e-4
    dYa = np.abs(dY.float().numpy().astype(np.float64))
    sabs_x = dYa @ np.abs(oracle.dequantize_groupwise(d["oc"], d["oh"], bits).astype(np.float64))
    bad = np.abs(gdx - odX) > 2.0 ** -8 * np.abs(odX) + 2.0 ** -8 * sabs_x
    assert not bad.any(), "dX: %d elements outside the bound" % bad.sum()
    sabs_w = dYa.T @ np.abs(oracle.dequantize_act(d["oq"], CLIP).astype(np.float64))
    bad = np.abs(gdw - odW) > 2.0 ** -12 * sabs_w
    assert not bad.any(), "dW: %d elements outside the bound" % bad.sum()


def test_backward_calls_on_two_streams_at_once(qb):
    """Two backward calls (QKV and FFN-up at 4096 tokens, each its own workspace) enqueued on two streams so that their
    launches compete for the CUs: inside a launch a workgroup waits for partial sums of workgroups dispatched before it,
    which must not depend on having the chip to itself.  Each result equals, bit for bit, the same call run alone."""
    T, bits = 4096, 3
    say("bwd on two streams")
    cases = []
    for i, (name, N, K) in enumerate([wl.BERT_BASE_LINEARS[0], wl.BERT_BASE_LINEARS[2]]):
        d = quantized_inputs(qb, N, K, T, bits, seed=700 + i)
        dY = wl.grad_output_bf16(T, N, seed=710 + i).to(DEV)
        ws = torch.empty(qb.qb_bwd_workspace_nbytes(T, N, K), dtype=torch.uint8, device=DEV)
        alone = qb.qb_qlinear_bwd_ste(dY, d["Xq"], CLIP, d["packed"], d["h"], bits, G, workspace=ws)
        cases.append(dict(d=d, dY=dY, ws=ws, alone=alone, N=N, K=K,
                          dX=torch.empty((T, K), dtype=torch.bfloat16, device=DEV),
                          dW=torch.empty((N, K), dtype=torch.float32, device=DEV)))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]   # default priority
    for rep in range(5):
        for c in cases:
            c["dX"].fill_(float("nan"))
            c["dW"].fill_(float("nan"))
        torch.cuda.synchronize()
        for c, st in zip(cases, streams):
            with torch.cuda.stream(st):
                for _ in range(3):
                    qb.qb_qlinear_bwd_ste(c["dY"], c["d"]["Xq"], CLIP, c["d"]["packed"], c["d"]["h"], bits, G, dX=c["dX"],
                                          dW=c["dW"], workspace=c["ws"])
        torch.cuda.synchronize()
        for c in cases:
            assert torch.equal(c["dX"].view(torch.int16), c["alone"][0].view(torch.int16))
            assert torch.equal(c["dW"].view(torch.int32), c["alone"][1].view(torch.int32))


def test_forward_next_to_another_streams_kernels(qb):
    """The step's shared forward launch on one stream while another stream runs backward calls (whose staging kernels
    keep the CUs' LDS busy): Y equals, bit for bit, the same call run alone.  A GEMM wavefront must not pass a step
    barrier while its LDS reads of the stage are still queued."""
    T, bits = 4096, 4
    say("fwd next to another stream's kernels")
    jobs = []
    for i, (name, N, K) in enumerate(wl.BERT_BASE_LINEARS):
        d = quantized_inputs(qb, N, K, T, bits, seed=800 + i)
        jobs.append(dict(Xq=d["Xq"], rs_x=d["rs_x"], clip=CLIP, packed=d["packed"], h=d["h"], rs_w=d["rs_w"], bits=bits,
                         groups=G, N=N, Y=torch.empty((T, N), dtype=torch.float32, device=DEV)))
    qb.qb_qlinear_fwd_batched(jobs)
    torch.cuda.synchronize()
    alone = [j["Y"].clone() for j in jobs]
    name, N, K = wl.BERT_BASE_LINEARS[0]
    b = quantized_inputs(qb, N, K, T, 3, seed=810)
    dY = wl.grad_output_bf16(T, N, seed=811).to(DEV)
    ws = torch.empty(qb.qb_bwd_workspace_nbytes(T, N, K), dtype=torch.uint8, device=DEV)
    dX = torch.empty((T, K), dtype=torch.bfloat16, device=DEV)
    dW = torch.empty((N, K), dtype=torch.float32, device=DEV)
    # the other stream also re-quantizes weights and activations; their results are checked as well
    Wd, Xd = b["W"].to(DEV), b["X"].to(DEV)
    q_alone = qb.qb_quantize_groupwise(Wd, 3, G)
    a_alone = qb.qb_quantize_act(Xd, CLIP)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()   # default priority
    for rep in range(4):
        for j in jobs:
            j["Y"].fill_(float("nan"))
        torch.cuda.synchronize()
        with torch.cuda.stream(s2):
            for _ in range(8):
                qb.qb_qlinear_bwd_ste(dY, b["Xq"], CLIP, b["packed"], b["h"], 3, G, dX=dX, dW=dW, workspace=ws)
                q_now = qb.qb_quantize_groupwise(Wd, 3, G)
                a_now = qb.qb_quantize_act(Xd, CLIP)
        with torch.cuda.stream(s1):
            for _ in range(6):
                qb.qb_qlinear_fwd_batched(jobs)
        torch.cuda.synchronize()
        for j, r in zip(jobs, alone):
            assert torch.equal(j["Y"].view(torch.int32), r.view(torch.int32))
        assert all(torch.equal(x.view(torch.uint8), y.view(torch.uint8)) for x, y in zip(q_now, q_alone))
        assert all(torch.equal(x.view(torch.uint8), y.view(torch.uint8)) for x, y in zip(a_now, a_alone))


# ---- batched activation quantizer ---------------------------------------------------------------------------------
def test_quantize_act_batched(qb):
    """The four inputs of a BERT-base layer at 4096 tokens plus ragged and tiny tensors (and two clips) in one call:
    codes and row sums bit for bit the oracle's, every output element written."""
    shapes = [(4096, 768, 6.0), (4096, 768, 6.0), (4096, 768, 3.0), (4096, 3072, 6.0), (1, 64, 6.0), (1023, 768, 2.5),
              (7, 1024, 6.0), (130, 4096, 1.0)]
    jobs, Xs = [], []
    for i, (T, K, clip) in enumerate(shapes):
        X = wl.activation(T, K, seed=900 + i)
        X[0, 0], X[-1, -1] = float("inf"), -float("inf")
        Xs.append(X)
        jobs.append(dict(X=X.to(DEV), clip=clip, Xq=torch.full((T, K), 77, dtype=torch.int8, device=DEV),
                         rs_x=torch.full((T,), -1, dtype=torch.int32, device=DEV)))
    say("act batched", len(jobs), "tensors")
    outs = qb.qb_quantize_act_batched(jobs)
    torch.cuda.synchronize()
    for (Xq, rs), X, (T, K, clip) in zip(outs, Xs, shapes):
        oq, orx = oracle.quantize_act(X.numpy(), clip)
        assert (Xq.cpu().numpy() == oq).all()
        assert (rs.cpu().numpy() == orx).all()
    assert qb.qb_quantize_act_batched([]) == []
    with pytest.raises(qb.QBError) as e:
        qb.qb_quantize_act_batched([jobs[0], dict(jobs[1], clip=-1.0)])
    assert e.value.status == 4


# ---- few tokens: the inference regime (batch x sequence of 1 ... 128 tokens) ---------------------------------------
@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("T", (1, 8, 64, 128))
def test_forward_few_tokens_bert_shapes(qb, bits, T):
    """BERT-base linears with 1 ... 128 tokens, alone and as one batched call of the layer's four linears: A4 bit for
    bit, Y within 1e-6, over the whole output."""
    jobs, refs = [], []
    for (name, N, K) in wl.BERT_BASE_LINEARS:
        say("fwd few tokens", (T, N, K), "bits", bits)
        d = quantized_inputs(qb, N, K, T, bits, seed=7 * N + K + T + bits)
        Y, A4 = qb.qb_qlinear_fwd(d["Xq"], d["rs_x"], CLIP, d["packed"], d["h"], d["rs_w"], bits, G, N, want_a4=True)
        Yp = qb.qb_qlinear_fwd(d["Xq"], d["rs_x"], CLIP, d["packed"], d["h"], d["rs_w"], bits, G, N)
        torch.cuda.synchronize()
        Yo, A4o, _ = oracle.qlinear_fwd(d["oq"], CLIP, d["oc"], d["oh"], bits)
        assert (A4.cpu().numpy() == A4o).all()
        assert_rel(Y.cpu().numpy(), Yo)
        assert torch.equal(Y, Yp)
        jobs.append(dict(Xq=d["Xq"], rs_x=d["rs_x"], clip=CLIP, packed=d["packed"], h=d["h"], rs_w=d["rs_w"], bits=bits,
                         groups=G, N=N))
        refs.append(Y)
    Ys = qb.qb_qlinear_fwd_batched(jobs)
    torch.cuda.synchronize()
    for Yb, Y in zip(Ys, refs):
        assert torch.equal(Yb, Y)


# ---- asymmetric ranges given by the caller -------------------------------------------------------------------------
@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", [(768, 768, 128), (2304, 768, 12), (768, 3072, 128), (6, 64, 6), (40, 192, 8), (1030, 64, 1)])
def test_quantize_given_asymmetric_ranges(qb, bits, shape):
    """Group ranges [lo, hi] from the caller (a 1 % / 99 % percentile band, the data's own [min, max] for one group and
    a degenerate range for another): codes, Delta, q0 and row sums bit for bit, then the forward through
    qb_qlinear_fwd_asym against the oracle."""
    N, K, groups = shape
    say("given asym ranges", shape, "bits", bits)
    W = wl.weight(N, K, seed=3 * N + K + bits) + 0.01
    Wg = W.reshape(groups, -1)
    lo = torch.quantile(Wg.double(), 0.01, dim=1).float()
    hi = torch.quantile(Wg.double(), 0.99, dim=1).float()
    lo[0], hi[0] = Wg[0].min(), Wg[0].max()
    if groups > 1:
        lo[-1] = hi[-1] = 0.02
    packed, delta, q0, rs_w = qb.qb_quantize_groupwise_asym_range(W.to(DEV), bits, lo.to(DEV), hi.to(DEV))
    codes = qb.qb_unpack_codes(packed, N, K, bits)
    torch.cuda.synchronize()
    oc, od, oq0, ors = oracle.quantize_groupwise_asym_range(W.numpy(), bits, lo.numpy(), hi.numpy())
    assert (codes.cpu().numpy() == oc).all()
    assert (delta.cpu().numpy().view(np.uint32) == od.view(np.uint32)).all()
    assert (q0.cpu().numpy().view(np.uint32) == oq0.view(np.uint32)).all()
    assert (rs_w.cpu().numpy() == ors).all()
    L = 2 ** bits - 1
    assert ((oc == 0) | (oc == L)).sum() > 0   # something was clamped
    T = 70
    X = wl.activation(T, K, seed=N + bits)
    Xq, rs_x = qb.qb_quantize_act(X.to(DEV), CLIP)
    Y, A4 = qb.qb_qlinear_fwd_asym(Xq, rs_x, CLIP, packed, delta, q0, rs_w, bits, groups, N, want_a4=True)
    torch.cuda.synchronize()
    oxq, _ = oracle.quantize_act(X.numpy(), CLIP)
    Yo, S = oracle.qlinear_fwd_asym(oxq, CLIP, oc, od, oq0, want_s=True)
    R = (2 * oxq.astype(np.int64) + 1).sum(1)
    hx = float(np.float32(CLIP) / np.float32(255.0))
    rows = N // groups
    mag = hx * (np.abs(od.astype(np.float64)).repeat(rows)[None, :] * np.abs(S) + np.abs(oq0.astype(np.float64)).repeat(rows)[None, :] * np.abs(R)[:, None])
    assert (np.abs(Y.cpu().numpy().astype(np.float64) - Yo) <= 1e-6 * mag).all()


def _check_quant_job(qb, job, out):
    packed, h, m, rs = out
    W = job["W"]
    N, K = W.shape
    oc, oh, om, ors = oracle.quantize_groupwise(W.cpu().numpy(), job["bits"], job["groups"])
    codes = qb.qb_unpack_codes(packed, N, K, job["bits"]).cpu().numpy()
    assert (codes == oc).all(), (N, K, job["bits"], job["groups"])
    assert (h.cpu().numpy().view(np.uint32) == oh.view(np.uint32)).all()
    assert (m.cpu().numpy().view(np.uint32) == om.view(np.uint32)).all()
    assert (rs.cpu().numpy() == ors).all()


def test_quantize_batched_work_items(qb):
    """The batched quantizer's work items: one, two or four groups per workgroup (teams of threads), groups whose
    size is no multiple of a team, group counts not divisible by four or two, weights parked in LDS (groups of more
    than 16384 weights in the 512-thread kernel), all three workgroup sizes, more jobs than one launch takes, and
    more items than resident workgroups (several items per workgroup).  Every output against the oracle, bit for bit."""
    mixes = {
        "256 threads": [(96, 64, 6), (64, 128, 64), (128, 64, 1), (70, 64, 10), (512, 192, 128)],
        "512 threads": [(768, 768, 128), (3072, 768, 128), (768, 3072, 128), (96, 192, 6), (2304, 768, 128),
                        (260, 640, 13), (640, 1024, 32)],
        "1024 threads": [(1024, 1024, 128), (4096, 1024, 128), (1024, 4096, 128), (62, 960, 2), (96, 64, 3)],
    }
    for name, shapes in mixes.items():
        jobs = []
        for rep in range(3):
            for i, (N, K, groups) in enumerate(shapes):
                bits = (2, 3, 4, 8)[(i + rep) % 4]
                gen = wl.weight_uniform if (i + rep) % 3 == 0 else wl.weight
                jobs.append({"W": gen(N, K, seed=1000 * rep + i).to(DEV), "bits": bits, "groups": groups})
        say("batched quantize work items,", name, len(jobs), "jobs")
        outs = qb.qb_quantize_groupwise_batched(jobs)
        torch.cuda.synchronize()
        for job, out in zip(jobs, outs):
            _check_quant_job(qb, job, out)
    # more jobs than one launch takes, many small groups: several items per resident workgroup
    jobs = [{"W": wl.weight(768, 768, seed=50 + i).to(DEV), "bits": (2, 3, 4, 8)[i % 4], "groups": 128} for i in range(70)]
    say("batched quantize work items, 70 small matrices")
    outs = qb.qb_quantize_groupwise_batched(jobs)
    torch.cuda.synchronize()
    for i in (0, 1, 2, 3, 47, 48, 69):
        _check_quant_job(qb, jobs[i], outs[i])
    # and a single small matrix (few items: one group per item)
    job = {"W": wl.weight(768, 768, seed=7).to(DEV), "bits": 3, "groups": 128}
    _check_quant_job(qb, job, qb.qb_quantize_groupwise_batched([job])[0])


def _shifted_weight(N, K, G, seed):
    """Weights whose groups sit at different offsets (what asymmetric ranges are for)."""
    W = wl.weight(N, K, seed=seed)
    rows = N // G
    off = torch.linspace(-0.05, 0.08, G).repeat_interleave(rows)[:, None]
    return (W + off).contiguous()


@pytest.mark.parametrize("bits", (2, 3, 4, 8))
@pytest.mark.parametrize("shape", [(300, 160, 192, 8), (1, 32, 64, 1), (129, 130, 320, 10), (513, 768, 768, 128),
                                   (2048, 1024, 128, 128), (2304, 1536, 128, 128), (4096, 768, 256, 128)])
def test_forward_asymmetric_ranges_with_per_token_scales(qb, bits, shape):
    """qb_qlinear_fwd_asym_dyn: asymmetric group ranges and one activation scale per token, through the register-staged
    kernel and both role-split layouts, ragged T and N, with and without bias; rows of very different magnitude and an
    all-zero row.  Y against the oracle within 1e-6 of h_x[t]*(Delta*|S| + |q0|*|R|), A4 bit for bit; a constant scale
    vector gives the fixed-clip call's bits."""
    T, N, K, G = shape
    say("fwd asym x per-token", shape, "bits", bits)
    W = _shifted_weight(N, K, G, seed=5 * N + K + bits)
    g = torch.Generator(device="cpu").manual_seed(T + 7 * K + bits)
    X = (wl.activation(T, K, seed=T + K + bits) * (0.05 + 4.0 * torch.rand(T, 1, generator=g))).contiguous()
    if T > 4:
        X[3] = 0.0
    bias = (0.3 * wl.activation(1, N, seed=13)[0]).contiguous()
    packed, delta, q0, rs_w = qb.qb_quantize_groupwise_asym(W.to(DEV), bits, G)
    Xq, rs_x, hx = qb.qb_quantize_act_dyn(X.to(DEV))
    oc, od, oq0, _ = oracle.quantize_groupwise_asym(W.numpy(), bits, G)
    oq, ors_x, ohx = oracle.quantize_act_dyn(X.numpy())
    assert (Xq.cpu().numpy() == oq).all() and (hx.cpu().numpy().view(np.uint32) == ohx.view(np.uint32)).all()
    L = 2 ** bits - 1
    xi = 2 * oq.astype(np.int64) + 1
    S = xi @ oc.astype(np.int64).T
    R = xi.sum(axis=1)[:, None]
    rows = N // G
    dn = np.repeat(od.astype(np.float64), rows)[None, :]
    zn = np.repeat(oq0.astype(np.float64), rows)[None, :]
    bound = 1e-6 * ohx.astype(np.float64)[:, None] * (dn * np.abs(S) + np.abs(zn) * np.abs(R))
    for b in (None, bias):
        Y, A4 = qb.qb_qlinear_fwd_asym_dyn(Xq, rs_x, hx, packed, delta, q0, rs_w, bits, G, N,
                                           bias=None if b is None else b.to(DEV), want_a4=True)
        torch.cuda.synchronize()
        assert (A4.cpu().numpy().astype(np.int64) == 2 * S - L * R).all()
        ref = oracle.qlinear_fwd_asym_dyn(oq, ohx, oc, od, oq0, bias=None if b is None else b.numpy(), openmp=True)
        extra = 0 if b is None else 1e-6 * np.abs(b.numpy())[None, :]
        assert (np.abs(Y.cpu().numpy().astype(np.float64) - ref) <= bound + extra + 1e-30).all()
        Y2 = qb.qb_qlinear_fwd_asym_dyn(Xq, rs_x, hx, packed, delta, q0, rs_w, bits, G, N, bias=None if b is None else b.to(DEV))
        torch.cuda.synchronize()
        assert torch.equal(Y2, Y)   # the timed path (no A4 output) gives the same bits
    # constant scales: the fixed-clip call, bit for bit
    Xs, rs_s = qb.qb_quantize_act(X.to(DEV), CLIP)
    const = torch.from_numpy(np.full(T, np.float32(CLIP) / np.float32(255.0), np.float32)).to(DEV)   # fl(clip/255), as the call forms it
    Ya = qb.qb_qlinear_fwd_asym_dyn(Xs, rs_s, const, packed, delta, q0, rs_w, bits, G, N, bias=bias.to(DEV))
    Yb = qb.qb_qlinear_fwd_asym(Xs, rs_s, CLIP, packed, delta, q0, rs_w, bits, G, N, bias=bias.to(DEV))
    torch.cuda.synchronize()
    assert torch.equal(Ya, Yb)


def test_forward_batched_few_token_jobs_share_launches(qb):
    """The inference regime: few-token problems of a batched call go through shared launches of the 32x64-tile kernel
    (one per bit-width and step width).  More jobs of one kind than a launch takes, all three step widths (K = 192,
    768, 3072), ragged T and N, with and without bias: every Y element by element against the oracle, pre-filled
    outputs fully written."""
    jobs, refs = [], []
    shapes = [(1, 768, 768), (8, 2304, 768), (64, 3072, 768), (128, 768, 3072), (33, 130, 192), (100, 96, 3072), (5, 64, 64)]
    case = 0
    for bits in BITS:
        for rep in range(3 if bits == 4 else 1):        # 21 jobs at 4 bits: more than one launch holds
            for (T, N, K) in shapes:
                groups = G if N % G == 0 else (N // 2 if N % 2 == 0 else 1)
                d = quantized_inputs(qb, N, K, T, bits, seed=31 * N + K + T + bits + 7 * rep, groups=groups)
                bias = wl.activation(1, N, seed=case)[0].contiguous() if case % 2 == 0 else None
                jobs.append(dict(Xq=d["Xq"], rs_x=d["rs_x"], clip=CLIP, packed=d["packed"], h=d["h"], rs_w=d["rs_w"], bits=bits,
                                 groups=groups, N=N, bias=None if bias is None else bias.to(DEV),
                                 Y=torch.full((T, N), float("nan"), dtype=torch.float32, device=DEV)))
                refs.append((d, bits, bias))
                case += 1
    say("fwd batched, few-token jobs:", len(jobs))
    Ys = qb.qb_qlinear_fwd_batched(jobs)
    torch.cuda.synchronize()
    for j, Yb, (d, bits, bias) in zip(jobs, Ys, refs):
        Yo, _, _ = oracle.qlinear_fwd(d["oq"], CLIP, d["oc"], d["oh"], bits)
        Yh = Yb.cpu().numpy().astype(np.float64)
        assert np.isfinite(Yh).all()
        if bias is not None:
            b = bias.numpy().astype(np.float64)[None, :]
            assert (np.abs(Yh - (Yo + b)) <= 1e-6 * np.abs(Yo) + 2.0 ** -23 * np.abs(Yo + b)).all()
        else:
            assert_rel(Yh, Yo)
        Y1 = qb.qb_qlinear_fwd(j["Xq"], j["rs_x"], CLIP, j["packed"], j["h"], j["rs_w"], bits, j["groups"], j["N"], bias=j["bias"])
        torch.cuda.synchronize()
        assert torch.equal(Yb, Y1)
