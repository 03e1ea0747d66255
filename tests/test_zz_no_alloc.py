"""ea_select_static (scratch in a static device array inside the library, no workspace argument,
no allocation) against ea_select on the same scores: identical indices, bit for bit, on two
calls in a row, the second on a smaller input (the array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest

from ea_inputs import CONFIGS
from oracle import ea_oracle as O
from tests import parity as P
import paper_2510_00636_amd as ea

pytestmark = pytest.mark.gpu


def _scores(B, H, n, seed):
    r = np.random.default_rng(seed)
    sc = np.exp(r.standard_normal((B, H, n))).astype(np.float32)
    sc[0, 0, ::5] = sc[0, 0, 0]                     # ties at the threshold's neighbourhood
    sc[-1, -1] = np.float32(0.25)                   # every score equal
    return sc


def test_select_static_matches_select_on_two_calls_in_a_row():
    import torch
    cfg = CONFIGS["c2"].with_(batch=2, n_kv_heads=3, n_q_heads=3)
    p = P.params_for(cfg)
    lib = ea.load_library()
    # first a long head (multi-launch path: global histograms and block counts in the scratch
    # array), then a shorter one of the same path, then one short enough for the one-launch path
    for n, n_keep in ((150000, 70001), (40000, 123), (5000, 2500)):
        sc = _scores(2, 3, n, n)
        want = P.run_select(cfg, sc, n_keep)
        scd = P.to_dev(sc)
        idx = torch.full((2, 3, n_keep), -1, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        # straight through the C ABI: no workspace pointer, no size
        rc = lib.ea_select_static(ctypes.byref(p), ctypes.c_void_p(scd.data_ptr()), n, n_keep,
                                  ctypes.c_void_p(idx.data_ptr()),
                                  ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0
        torch.cuda.synchronize()
        got = idx.cpu().numpy()
        assert np.array_equal(got, want), (n, n_keep)
        assert np.array_equal(got.astype(np.int64), O.select(sc.astype(np.float64), n_keep))


def test_select_static_rejects_sizes_beyond_its_array():
    import torch
    lib = ea.load_library()
    dummy = torch.zeros(64, dtype=torch.float32, device="cuda")
    out = torch.zeros(64, dtype=torch.int32, device="cuda")
    big_units = ea.make_params(65, 1, 1, 128, ea.EA_BF16)
    ok = ea.make_params(1, 1, 1, 128, ea.EA_BF16)
    VP = ctypes.c_void_p
    assert lib.ea_select_static(ctypes.byref(big_units), VP(dummy.data_ptr()), 8, 4, VP(out.data_ptr()), None) == 2
    assert lib.ea_select_static(ctypes.byref(ok), VP(dummy.data_ptr()), (1 << 20) + 1, 4, VP(out.data_ptr()), None) == 2
    assert lib.ea_select_static(ctypes.byref(ok), VP(dummy.data_ptr()), 8, 9, VP(out.data_ptr()), None) == 1
    torch.cuda.synchronize()
    assert int(out.abs().sum()) == 0            # nothing was launched
