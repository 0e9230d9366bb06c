"""The injection entry point that allocates nothing, called through the C ABI, against
codenet_inject on the same inputs: identical bits, on two calls in a row of which the second is
smaller (fewer faults, a smaller batch), then on the stored weights."""
import ctypes

import numpy as np
import pytest

from paper_1903_01042_amd import workloads as WL

pytestmark = pytest.mark.gpu


def test_injection_without_allocation_matches_codenet_inject():
    import torch
    from paper_1903_01042_amd import binding as B
    dev = torch.device("cuda:0")
    m, n, r = 4, 3, 2
    n_out, n_in = 200, 150
    P_r, P_c = WL.vandermonde_like(m, r), WL.vandermonde_like(n, r)
    W = torch.from_numpy(WL.layer_weights(n_out, n_in)).to(dev)
    layers = [B.CodedLayer(W, P_r, P_c, dtype=dt, max_batch=96) for dt in (B.F32, B.BF16_F32ACC)]
    lib = B.load_library()
    for lay in layers:
        for call, (b, faults) in enumerate((
                (96, [WL.make_fault(WL.PHASE_FWD, i, i % n, 7) for i in (0, 2, 5, 3, 2)]),      # two on block-row 2
                (17, [WL.make_fault(WL.PHASE_FWD, 4, 1, 8)]))):
            print("no-alloc injection: forward outputs, call", call, "batch", b, "faults", len(faults), flush=True)
            X = torch.from_numpy(WL.normal((b, n_in), 50 + call)).to(dev)
            ref = lay.forward(X)
            got = ref.clone()
            lay.inject(faults, ref)
            # straight through the C ABI: pointers and sizes only
            arr = B.pack_faults(faults)
            rc = lib.codenet_inject_noalloc(lay._h, arr, len(faults), ctypes.c_void_p(got.data_ptr()), b,
                                            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
            assert rc == 0
            torch.cuda.synchronize()
            assert torch.equal(ref, got)
            assert not torch.equal(ref, lay.forward(X))            # the faults did change something
        # backward outputs, sparse law, then stored weights: the same on a twin layer
        D = torch.from_numpy(WL.normal((40, n_out), 60)).to(dev)
        ref = lay.backward(D)
        got = ref.clone()
        fb = [WL.make_fault(WL.PHASE_BWD, 1, 4, 9), WL.make_fault(WL.PHASE_BWD, 0, 0, 9, lo=-5.0, hi=5.0,
                                                                 mode=WL.MODE_SPARSE_ABS, density=0.05)]
        lay.inject(fb, ref)
        lay.inject(fb, got, noalloc=True)
        assert torch.equal(ref, got)
    twin = B.CodedLayer(W, P_r, P_c, dtype=B.BF16_F32ACC, max_batch=96)
    fw = [WL.make_fault(WL.PHASE_WEIGHT, 1, 2, 3), WL.make_fault(WL.PHASE_WEIGHT, 5, 0, 3)]
    layers[1].inject(fw)
    twin.inject(fw, noalloc=True)
    assert torch.equal(layers[1].export_coded(), twin.export_coded())
    X = torch.from_numpy(WL.normal((8, n_in), 70)).to(dev)
    assert torch.equal(layers[1].forward(X), twin.forward(X))      # the bf16 copy was refreshed alike
    # more faults than the scratch array holds partial sums for
    many = B.pack_faults([WL.make_fault(WL.PHASE_FWD, 0, 0, 1)] * (B.MAX_FAULTS + 1))
    out = layers[0].forward(X)
    assert lib.codenet_inject_noalloc(layers[0]._h, many, B.MAX_FAULTS + 1, ctypes.c_void_p(out.data_ptr()), 8, None) == B.E_SHAPE
    assert lib.codenet_inject_noalloc(None, many, 1, None, 8, None) == B.E_NULL
    for lay in layers + [twin]:
        lay.destroy()
