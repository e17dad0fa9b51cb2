"""small_network_run_static (the entry point for callers that cannot allocate: the layer workspace is an array
inside the library's device image) against small_network_run_opt with a caller-provided workspace, through the C ABI."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2303_04769_amd as S
import workloads as WL
from oracle import oracle as O
from gpu_util import CANARY, DEV, Guarded, assert_bits, assert_close, dev

pytestmark = pytest.mark.gpu


def _both(name, idx, N, flags, seed):
    """Blocked outputs of the workspace-argument entry point and of the allocation-free one, both through ctypes."""
    from paper_2303_04769_amd import binding as B
    lib = B.load()
    net = getattr(WL, name)()
    x, ws = WL.network_tensors(net, N, seed)
    pn = S.PackedNetwork(net, ws, DEV)
    xb = pn.pack_input(dev(x))
    table = pn.table
    nbytes = S.small_network_workspace(table, N, net.C0, net.H0, net.W0)
    wsp = torch.empty(max(nbytes, 256) // 4, dtype=torch.float32, device=DEV)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    g0, g1 = Guarded(pn.out_elems(N)), Guarded(pn.out_elems(N))
    rc = lib.small_network_run_opt(table, len(table), C.c_void_p(xb.data_ptr()), C.c_void_p(g0.t.data_ptr()),
                                   C.c_void_p(wsp.data_ptr()), nbytes, N, net.C0, net.H0, net.W0, flags, stream)
    assert rc == 0
    before = torch.cuda.memory_allocated()
    rc = lib.small_network_run_static(table, len(table), C.c_void_p(xb.data_ptr()), C.c_void_p(g1.t.data_ptr()), N,
                                      net.C0, net.H0, net.W0, flags, stream)
    assert rc == 0
    assert torch.cuda.memory_allocated() == before
    a, b = g0.check(), g1.check()
    L = net.layers[-1]
    ref = O.run_network(net, x, ws)
    got = O.unpack(b, (N, L.Co, L.Ho, L.Wo), L.Cob).reshape(ref.shape)
    K = max([l.Ci * l.kh * l.kw for l in net.layers if l.op in ("conv", "dense")] + [9])
    return a, b, got, ref, K, nbytes


@pytest.mark.parametrize("name,idx,N1,N2", [("residual_cnn", 2, 64, 5), ("dsep_cnn", 3, 40, 3), ("audio_cnn", 4, 700, 33)])
def test_static_workspace_run_matches_the_workspace_argument_run(name, idx, N1, N2):
    """Two calls in a row on the one built-in array, the second with a smaller batch (the array still holds the first
    call's tensors): bit for bit the results of the existing entry point, and the oracle's within the stated
    tolerance. Layer-by-layer launches, so that the workspace slots really carry the tensors."""
    for N in (N1, N2):
        a, b, got, ref, K, nbytes = _both(name, idx, N, S.SMALL_RUN_RESIDENT_OFF, 8800 + N)
        assert 0 < nbytes <= S.STATIC_WORKSPACE_BYTES
        assert_bits(b, a, f"{name} N={N}: built-in array vs workspace argument")
        assert_close(got, ref, K, f"{name} N={N}: built-in array vs oracle")


def test_static_workspace_run_with_default_flags_and_plain_boundaries():
    """Default planning (image-resident run at batch 200) and the plain input / output options go through as well."""
    a, b, got, ref, K, _ = _both("residual_cnn", 2, 200, 0, 8700)
    assert_bits(b, a, "default flags")
    assert_close(got, ref, K, "default flags vs oracle")


def test_static_workspace_run_refuses_what_does_not_fit():
    """A batch whose workspace exceeds the array: error 9 (clear message), nothing written; bad flags: error 2."""
    from paper_2303_04769_amd import binding as B
    lib = B.load()
    net = WL.dsep_cnn()
    N = 1024
    x, ws = WL.network_tensors(net, 1, 1)
    pn = S.PackedNetwork(net, ws, DEV)
    assert S.small_network_workspace(pn.table, N, net.C0, net.H0, net.W0) > S.STATIC_WORKSPACE_BYTES
    xb = torch.zeros(N * net.C0 * net.H0 * net.W0, dtype=torch.float32, device=DEV)
    g = Guarded(pn.out_elems(N))
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = lib.small_network_run_static(pn.table, len(pn.table), C.c_void_p(xb.data_ptr()), C.c_void_p(g.t.data_ptr()), N,
                                      net.C0, net.H0, net.W0, 0, stream)
    assert rc == 9 and b"SMALL_STATIC_WORKSPACE_BYTES" in lib.small_strerror(rc)
    assert (g.check() == np.float32(CANARY)).all()
    rc = lib.small_network_run_static(pn.table, len(pn.table), C.c_void_p(xb.data_ptr()), C.c_void_p(g.t.data_ptr()), 2,
                                      net.C0, net.H0, net.W0, 64, stream)
    assert rc == 2
