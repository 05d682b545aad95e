"""The backward entry point that allocates nothing (its staging area is a fixed array of the library): called through
the C ABI, it must give bit for bit what qb_qlinear_bwd_ste gives with a caller-provided workspace -- on two calls in
a row, the second with a smaller input (the shared array still holds the first call's contents), and must refuse
shapes beyond its fixed size."""
import ctypes

import numpy as np
import pytest
import torch

from paper_1909_05840_amd import workloads as wl

pytestmark = pytest.mark.gpu
CLIP = 6.0
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


def one_case(qb, T, N, K, G, bits, seed):
    say("no-alloc backward", (T, N, K, G), "bits", bits)
    lib = qb.load_library()
    W = wl.weight(N, K, seed=seed).to(DEV)
    X = wl.activation(T, K, seed=seed + 1).to(DEV)
    dY = wl.grad_output_bf16(T, N, seed=seed + 2).to(DEV)
    packed, h, m, rs_w = qb.qb_quantize_groupwise(W, bits, G)
    Xq, rs_x = qb.qb_quantize_act(X, CLIP)
    # the existing entry point, its workspace filled with a pattern that must not matter
    ws = torch.full((max(qb.qb_bwd_workspace_nbytes(T, N, K), 256),), 0xA5, dtype=torch.uint8, device=DEV)
    dX_ref, dW_ref = qb.qb_qlinear_bwd_ste(dY, Xq, CLIP, packed, h, bits, G, workspace=ws)
    # the new one, straight through the C ABI
    dX = torch.full((T, K), float("nan"), dtype=torch.bfloat16, device=DEV)
    dW = torch.full((N, K), float("nan"), dtype=torch.float32, device=DEV)
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    vp = ctypes.c_void_p
    rc = lib.qb_qlinear_bwd_ste_static(vp(dY.data_ptr()), vp(Xq.data_ptr()), ctypes.c_float(CLIP), vp(packed.data_ptr()),
                                       vp(h.data_ptr()), bits, G, T, N, K, vp(dX.data_ptr()), vp(dW.data_ptr()), st)
    assert rc == 0, qb.qb_status_string(rc)
    torch.cuda.synchronize()
    assert torch.equal(dX.view(torch.int16), dX_ref.view(torch.int16)), "dX differs from qb_qlinear_bwd_ste"
    assert torch.equal(dW.view(torch.int32), dW_ref.view(torch.int32)), "dW differs from qb_qlinear_bwd_ste"
    # one output only (compared with the existing entry point called the same way: which outputs a call computes
    # decides how its workgroups share the contraction, and with that the order of the fp32 additions)
    dX2_ref, _ = qb.qb_qlinear_bwd_ste(dY, Xq, CLIP, packed, h, bits, G, want_dw=False, workspace=ws)
    dX2 = torch.full((T, K), float("nan"), dtype=torch.bfloat16, device=DEV)
    rc = lib.qb_qlinear_bwd_ste_static(vp(dY.data_ptr()), vp(Xq.data_ptr()), ctypes.c_float(CLIP), vp(packed.data_ptr()),
                                       vp(h.data_ptr()), bits, G, T, N, K, vp(dX2.data_ptr()), None, st)
    assert rc == 0
    torch.cuda.synchronize()
    assert torch.equal(dX2.view(torch.int16), dX2_ref.view(torch.int16))


def test_static_backward_matches_workspace_backward_twice_in_a_row(qb):
    # a BERT-base linear at configuration-3 size (58.5 MiB of staging), then smaller ones with ragged
    # sizes that leave most of the array holding the first call's bytes
    one_case(qb, 4096, 768, 3072, 128, 3, seed=41)
    one_case(qb, 300, 160, 192, 8, 4, seed=42)
    one_case(qb, 1500, 768, 768, 128, 2, seed=43)
    one_case(qb, 65, 6, 64, 6, 8, seed=44)


def test_static_backward_refuses_what_does_not_fit(qb):
    lib = qb.load_library()
    T, N, K = 12288, 3072, 768   # needs 118.5 MiB of staging
    assert qb.qb_bwd_workspace_nbytes(T, N, K) > (60 << 20)
    dX = torch.full((8,), 3.0, dtype=torch.bfloat16, device=DEV)
    vp = ctypes.c_void_p
    one = vp(dX.data_ptr())   # never dereferenced: the call is refused on the host
    rc = lib.qb_qlinear_bwd_ste_static(one, one, ctypes.c_float(CLIP), one, one, 4, 128, T, N, K, one, None,
                                       vp(torch.cuda.current_stream().cuda_stream))
    assert rc == 5   # QB_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert (dX.float() == 3.0).all()
