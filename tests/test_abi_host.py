"""Host-side checks of the C ABI that need no GPU: every declared symbol is exported, the pure
host functions are right, and invalid arguments are refused before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_1909_05840_amd as qb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(qb.LIB_PATH):
        from paper_1909_05840_amd import build
        build.build()
    return qb.load_library()


def test_header_symbols_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "qbert.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(qb_[a-z0-9_]+)\s*\(", text))
    assert names == set(qb.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_packed_nbytes_follows_paper_size_arithmetic(lib):
    for bits in (2, 3, 4, 8):
        for N, K in ((768, 768), (2304, 768), (3072, 768), (768, 3072), (1024, 4096), (4096, 1024)):
            assert qb.qb_packed_nbytes(N, K, bits) == N * K * bits // 8
        assert qb.qb_packed_nbytes(6, 64, bits) == 32 * 64 * bits // 8  # rows padded to a block of 32
    assert qb.qb_packed_nbytes(768, 768, 5) == 0
    assert qb.qb_packed_nbytes(768, 100, 4) == 0
    assert qb.qb_packed_nbytes(0, 64, 4) == 0
    # one BERT-base encoder layer's matrices at 2 bits: 7,077,888 * 2 / 8 bytes
    total = sum(qb.qb_packed_nbytes(N, K, 2) for _, N, K in qb.workloads.BERT_BASE_LINEARS)
    assert total == 7077888 * 2 // 8


def test_workspace_size(lib):
    assert qb.qb_bwd_workspace_nbytes(4096, 768, 768) > 0
    assert qb.qb_bwd_workspace_nbytes(4096, 768, 700) == 0
    assert qb.qb_bwd_workspace_nbytes(0, 768, 768) == 0


def test_general_workspace_query(lib):
    bwd = qb.qb_bwd_workspace_nbytes(4096, 768, 3072)
    assert qb.qb_workspace_nbytes(qb.binding.QB_OP_QLINEAR_BWD_STE, 4096, 768, 3072, 3) == bwd
    assert qb.qb_workspace_nbytes(qb.binding.QB_OP_QLINEAR_BWD_STE, 4096, 768, 3072, 5) == 0
    assert qb.qb_workspace_nbytes(qb.binding.QB_OP_POWER_ITERATION, 0, 0, 0, 0) == 4 * lib.qb_power_iteration_scratch_floats()
    for op in (qb.binding.QB_OP_QUANTIZE_GROUPWISE, qb.binding.QB_OP_QUANTIZE_ACT, qb.binding.QB_OP_QLINEAR_FWD,
               qb.binding.QB_OP_EMBEDDING, 99):
        assert qb.qb_workspace_nbytes(op, 4096, 768, 3072, 4) == 0


def test_batched_calls_and_the_static_backward_refuse_bad_arguments_on_the_host(lib):
    P = 0x1000
    fj = qb.binding._FwdJob(P, P, 6.0, P, P, P, 4, 128, 4096, 768, 768, None, P)
    arr = (qb.binding._FwdJob * 2)(fj, fj)
    assert lib.qb_qlinear_fwd_batched(arr, 0, None) == 0
    assert lib.qb_qlinear_fwd_batched(None, 2, None) == 1
    arr[1].bits = 7
    assert lib.qb_qlinear_fwd_batched(arr, 2, None) == 2
    arr[1].bits = 4
    arr[1].K = 100
    assert lib.qb_qlinear_fwd_batched(arr, 2, None) == 3
    arr[1].K = 768
    arr[1].clip = 0.0
    assert lib.qb_qlinear_fwd_batched(arr, 2, None) == 4
    aj = qb.binding._ActJob(P, 16, 64, 6.0, P, P)
    aarr = (qb.binding._ActJob * 2)(aj, aj)
    assert lib.qb_quantize_act_batched(aarr, 0, None) == 0
    aarr[1].K = 65
    assert lib.qb_quantize_act_batched(aarr, 2, None) == 3
    aarr[1].K = 64
    aarr[1].Xq = None
    assert lib.qb_quantize_act_batched(aarr, 2, None) == 1
    vp, cf = ctypes.c_void_p, ctypes.c_float
    # the static backward: shape and size checks come before the device is touched
    assert lib.qb_qlinear_bwd_ste_static(vp(P), vp(P), cf(6.0), vp(P), vp(P), 4, 128, 12288, 3072, 768, vp(P), None, None) == 5
    assert lib.qb_qlinear_bwd_ste_static(vp(P), vp(P), cf(6.0), vp(P), vp(P), 4, 128, 4096, 768, 100, vp(P), None, None) == 3
    # embedding tables whose row count exceeds the grid's second dimension
    assert lib.qb_embedding_quantize_bits(vp(P), 3000000, 64, 8, 8, vp(P), vp(P), vp(P), None) == 3


def test_status_strings(lib):
    seen = {qb.qb_status_string(i) for i in range(7)}
    assert len(seen) == 7 and "unknown" not in " ".join(seen)
    assert "unknown" in qb.qb_status_string(99)


def test_invalid_arguments_are_refused_on_the_host(lib):
    """Nothing is launched for these calls, so dummy non-null pointers are safe."""
    P = ctypes.c_void_p(0x1000)
    NULL = None
    f = ctypes.c_float
    # quantize_groupwise(W,N,K,bits,groups,packed,h,m,rs_w,stream)
    assert lib.qb_quantize_groupwise(NULL, 768, 768, 4, 128, P, P, P, P, NULL) == 1
    assert lib.qb_quantize_groupwise(P, 768, 768, 5, 128, P, P, P, P, NULL) == 2
    assert lib.qb_quantize_groupwise(P, 768, 768, 4, 100, P, P, P, P, NULL) == 3   # 768 % 100
    assert lib.qb_quantize_groupwise(P, 768, 760, 4, 128, P, P, P, P, NULL) == 3   # K % 64
    assert lib.qb_quantize_groupwise(P, 768, 65536, 4, 128, P, P, P, P, NULL) == 3  # K too large
    assert lib.qb_quantize_groupwise(P, 0, 768, 4, 128, P, P, P, P, NULL) == 3
    # quantize_act(X,T,K,clip,Xq,rs_x,stream)
    assert lib.qb_quantize_act(P, 16, 64, f(6.0), NULL, P, NULL) == 1
    assert lib.qb_quantize_act(P, 16, 64, f(0.0), P, P, NULL) == 4
    assert lib.qb_quantize_act(P, 16, 64, f(float("inf")), P, P, NULL) == 4
    assert lib.qb_quantize_act(P, 16, 64, f(float("nan")), P, P, NULL) == 4
    assert lib.qb_quantize_act(P, 16, 65, f(6.0), P, P, NULL) == 3
    # qlinear_fwd(Xq,rs_x,clip,packed,h,rs_w,bits,groups,T,N,K,bias,Y,A4,stream)
    assert lib.qb_qlinear_fwd(P, P, f(6.0), P, P, P, 4, 128, 16, 768, 768, NULL, NULL, NULL, NULL) == 1
    assert lib.qb_qlinear_fwd(P, P, f(6.0), P, P, P, 7, 128, 16, 768, 768, NULL, P, NULL, NULL) == 2
    assert lib.qb_qlinear_fwd(P, P, f(6.0), P, P, P, 4, 128, 16, 770, 768, NULL, P, NULL, NULL) == 3
    assert lib.qb_qlinear_fwd(P, P, f(-1.0), P, P, P, 4, 128, 16, 768, 768, NULL, P, NULL, NULL) == 4
    # qlinear_fwd_q8(Xq,rs_x,clip,packed,h,rs_w,bits,groups,T,N,K,bias,act,clip_out,Yq,rs_y,stream)
    assert lib.qb_qlinear_fwd_q8(P, P, f(6.0), P, P, P, 4, 128, 16, 768, 768, NULL, 0, f(6.0), NULL, P, NULL) == 1
    assert lib.qb_qlinear_fwd_q8(P, P, f(6.0), P, P, P, 5, 128, 16, 768, 768, NULL, 0, f(6.0), P, P, NULL) == 2
    assert lib.qb_qlinear_fwd_q8(P, P, f(6.0), P, P, P, 4, 128, 16, 768, 192, NULL, 0, f(6.0), P, P, NULL) == 3  # K % 128
    assert lib.qb_qlinear_fwd_q8(P, P, f(6.0), P, P, P, 4, 128, 16, 768, 768, NULL, 2, f(6.0), P, P, NULL) == 3  # act
    assert lib.qb_qlinear_fwd_q8(P, P, f(6.0), P, P, P, 4, 128, 16, 768, 768, NULL, 0, f(0.0), P, P, NULL) == 4
    # qlinear_bwd_ste(dY,Xq,clip,packed,h,bits,groups,T,N,K,dX,dW,workspace,stream)
    assert lib.qb_qlinear_bwd_ste(P, P, f(6.0), P, P, 4, 128, 16, 768, 768, P, P, NULL, NULL) == 5
    assert lib.qb_qlinear_bwd_ste(P, P, f(6.0), P, P, 4, 128, 16, 768, 768, P, P, ctypes.c_void_p(0x1010), NULL) == 5
    assert lib.qb_qlinear_bwd_ste(P, NULL, f(6.0), P, P, 4, 128, 16, 768, 768, P, P, P, NULL) == 1
    assert lib.qb_qlinear_bwd_ste(P, P, f(6.0), P, P, 4, 128, 16, 768, 768, NULL, NULL, NULL, NULL) == 0  # nothing asked
    # qlinear_bwd_ste_masked(dY,Xq,clip,packed,h,bits,groups,T,N,K,X,W,m,dX,dW,workspace,stream)
    assert lib.qb_qlinear_bwd_ste_masked(P, P, f(6.0), P, P, 4, 128, 16, 768, 768, P, P, NULL, P, P, P, NULL) == 1  # W without m
    assert lib.qb_qlinear_bwd_ste_masked(P, P, f(6.0), P, P, 4, 128, 16, 768, 768, P, NULL, P, P, P, P, NULL) == 1
    assert lib.qb_qlinear_bwd_ste_masked(P, P, f(6.0), P, P, 5, 128, 16, 768, 768, P, P, P, P, P, P, NULL) == 2
    assert lib.qb_qlinear_bwd_ste_masked(P, P, f(6.0), P, P, 4, 128, 16, 768, 768, P, P, P, P, P, NULL, NULL) == 5
    assert lib.qb_qlinear_bwd_ste_masked(P, P, f(6.0), P, P, 4, 128, 16, 768, 768, P, P, P, NULL, NULL, NULL, NULL) == 0
    # batched quantize: host array of descriptors, every job checked before any launch
    from paper_1909_05840_amd.binding import _QuantJob
    good = _QuantJob(0x1000, 768, 768, 4, 128, 0x1000, 0x1000, 0x1000, 0x1000)
    bad_bits = _QuantJob(0x1000, 768, 768, 6, 128, 0x1000, 0x1000, 0x1000, 0x1000)
    bad_null = _QuantJob(0x1000, 768, 768, 4, 128, 0, 0x1000, 0x1000, 0x1000)
    arr = (_QuantJob * 2)(good, bad_bits)
    assert lib.qb_quantize_groupwise_batched(arr, 2, NULL) == 2
    arr = (_QuantJob * 2)(good, bad_null)
    assert lib.qb_quantize_groupwise_batched(arr, 2, NULL) == 1
    assert lib.qb_quantize_groupwise_batched(arr, 0, NULL) == 0
    assert lib.qb_quantize_groupwise_batched(arr, -1, NULL) == 3
    assert lib.qb_quantize_groupwise_batched(None, 1, NULL) == 1
    # unpack / embedding
    assert lib.qb_unpack_codes(P, 768, 768, 1, P, NULL) == 2
    assert lib.qb_embedding_quantize(P, 100, 1024, 100, P, P, P, NULL) == 3   # 1024 % 100
    assert lib.qb_embedding_gather(P, P, 100, 1024, 128, P, 0, P, NULL) == 0  # empty lookup
    assert lib.qb_embedding_gather(P, P, 100, 1024, 128, P, -1, P, NULL) == 3
    # quantize_groupwise_clip(W,N,K,bits,groups,m_in,packed,h,rs_w,stream)
    assert lib.qb_quantize_groupwise_clip(P, 768, 768, 4, 128, NULL, P, P, P, NULL) == 1
    assert lib.qb_quantize_groupwise_clip(P, 768, 768, 5, 128, P, P, P, P, NULL) == 2
    assert lib.qb_quantize_groupwise_clip(P, 770, 768, 4, 128, P, P, P, P, NULL) == 3
    # quantize_act_dyn(X,T,K,Xq,rs_x,hx,stream), qlinear_fwd_dyn(Xq,rs_x,hx,packed,h,rs_w,bits,groups,T,N,K,bias,Y,A4,stream)
    assert lib.qb_quantize_act_dyn(P, 16, 64, P, P, NULL, NULL) == 1
    assert lib.qb_quantize_act_dyn(P, 16, 65, P, P, P, NULL) == 3
    # quantize_groupwise_asym(W,N,K,bits,groups,packed,delta,q0,rs_w,stream)
    assert lib.qb_quantize_groupwise_asym(P, 768, 768, 4, 128, P, P, NULL, P, NULL) == 1
    assert lib.qb_quantize_groupwise_asym(P, 768, 768, 7, 128, P, P, P, P, NULL) == 2
    assert lib.qb_quantize_groupwise_asym(P, 768, 768, 4, 100, P, P, P, P, NULL) == 3
    # qlinear_fwd_asym(Xq,rs_x,clip,packed,delta,q0,rs_w,bits,groups,T,N,K,bias,Y,A4,stream)
    assert lib.qb_qlinear_fwd_asym(P, P, f(6.0), P, P, NULL, P, 4, 128, 16, 768, 768, NULL, P, NULL, NULL) == 1
    assert lib.qb_qlinear_fwd_asym(P, P, f(6.0), P, P, P, P, 5, 128, 16, 768, 768, NULL, P, NULL, NULL) == 2
    assert lib.qb_qlinear_fwd_asym(P, P, f(6.0), P, P, P, P, 4, 128, 16, 768, 800, NULL, P, NULL, NULL) == 3
    assert lib.qb_qlinear_fwd_asym(P, P, f(-1.0), P, P, P, P, 4, 128, 16, 768, 768, NULL, P, NULL, NULL) == 4
    # qlinear_bwd_ste_asym(dY,Xq,clip,packed,delta,q0,bits,groups,T,N,K,dX,dW,workspace,stream)
    assert lib.qb_qlinear_bwd_ste_asym(P, P, f(6.0), P, P, NULL, 4, 128, 16, 768, 768, P, P, P, NULL) == 1
    assert lib.qb_qlinear_bwd_ste_asym(P, P, f(6.0), P, P, P, 4, 128, 16, 768, 768, P, P, NULL, NULL) == 5
    # quantize_act_dyn_tensor(X,T,K,Xq,rs_x,hx,c,stream)
    assert lib.qb_quantize_act_dyn_tensor(P, 16, 64, P, P, P, NULL, NULL) == 1
    assert lib.qb_quantize_act_dyn_tensor(P, 0, 64, P, P, P, P, NULL) == 3
    assert lib.qb_quantize_act_dyn_tensor(P, 16, 65, P, P, P, P, NULL) == 3
    assert lib.qb_qlinear_fwd_dyn(P, P, NULL, P, P, P, 4, 128, 16, 768, 768, NULL, P, NULL, NULL) == 1
    assert lib.qb_qlinear_fwd_dyn(P, P, P, P, P, P, 6, 128, 16, 768, 768, NULL, P, NULL, NULL) == 2
    assert lib.qb_qlinear_fwd_dyn(P, P, P, P, P, P, 4, 128, 16, 770, 768, NULL, P, NULL, NULL) == 3
    # embedding_quantize_bits(E,V,d,bits,groups,codes,h,m,stream), embedding_gather_bits(codes,h,V,d,bits,groups,ids,n,out,stream)
    assert lib.qb_embedding_quantize_bits(P, 100, 1024, 3, 128, P, P, P, NULL) == 2
    assert lib.qb_embedding_quantize_bits(P, 100, 1024, 4, 128, NULL, P, P, NULL) == 1
    assert lib.qb_embedding_quantize_bits(P, 100, 1000, 4, 125, P, P, P, NULL) == 3
    assert lib.qb_embedding_gather_bits(P, P, 100, 1024, 2, 128, P, 4, P, NULL) == 2
    assert lib.qb_embedding_gather_bits(P, P, 100, 1024, 4, 128, P, 0, P, NULL) == 0


def test_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_1909_05840_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                src = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in src and "from oracle" not in src and "qbert_oracle" not in src, fn


def test_sensitivity_host_functions_against_eq2():
    """Eq. 2 and the ranking run on the host: checked here against the oracle and hand-worked values, plus the
    argument errors of the device-side power iteration (no launch happens for those)."""
    import numpy as np
    from oracle import sensitivity_omega, rank_by_sensitivity
    lam = np.array([[1.0, 3.0], [-1.0, -3.0], [2.0, 2.0], [-4.0, 4.0]], np.float32)
    om = qb.qb_sensitivity_omega(lam)
    assert np.allclose(om, [3.0, 3.0, 2.0, 4.0], rtol=1e-7)
    assert qb.qb_rank_by_sensitivity(om).tolist() == [3, 0, 1, 2]
    r = np.random.default_rng(3)
    lam = r.normal(1.0, 5.0, (12, 10)).astype(np.float32)        # 12 encoder layers, 10 runs (Sec. 4)
    om = qb.qb_sensitivity_omega(lam)
    assert np.allclose(om, sensitivity_omega(lam), rtol=1e-6)
    assert (qb.qb_rank_by_sensitivity(om) == rank_by_sensitivity(om)).all()
    lib = qb.load_library()
    P, NULL = ctypes.c_void_p(0x1000), None
    cb = qb.binding.HV_FN(lambda ctx, v, out, stream: 0)
    assert lib.qb_power_iteration(cb, NULL, 100, 5, P, P, P, NULL, NULL) == 1
    assert lib.qb_power_iteration(cb, NULL, 0, 5, P, P, P, P, NULL) == 3
    assert lib.qb_power_iteration(cb, NULL, 100, 0, P, P, P, P, NULL) == 3
    assert lib.qb_sensitivity_omega(NULL, 3, 3, P) == 1
    assert lib.qb_sensitivity_omega(P, 0, 3, P) == 3
    assert lib.qb_rank_by_sensitivity(P, 0, P) == 3
    assert lib.qb_power_iteration_scratch_floats() >= 2
    # probe_mfma_i8(workgroups,iters,sink,stream)
    assert lib.qb_probe_mfma_i8(512, 100, NULL, NULL) == 1
    assert lib.qb_probe_mfma_i8(0, 100, P, NULL) == 3
    assert lib.qb_probe_mfma_i8(512, 0, P, NULL) == 3

