"""cocodiff_vmajor_select_static (no workspace argument, nothing allocated: the flag words live in a library-owned
device array) against cocodiff_vmajor_select, through the C ABI, bit for bit; two calls in a row on the shared array,
the second on a smaller input."""
import numpy as np
import pytest

import paper_2604_14561_amd as cd
from parity_util import dev_empty, to_dev, to_host_bits
from synth import f32_to_bf16_bits, perturb_tiles

pytestmark = pytest.mark.gpu


def _both(S, N, W, T, n_changed, seed, tau=1e-3, cap=None):
    import torch
    rng = np.random.default_rng(seed)
    NT = N // T
    cap = NT if cap is None else cap
    cur = f32_to_bf16_bits(rng.standard_normal((S, N, W)).astype(np.float32))
    prev, changed = perturb_tiles(cur, 1, T, n_changed, rng, sigma=0.05)
    cur_d, prev_d = to_dev(cur), to_dev(prev)
    outs = []
    for static in (False, True):
        flags, idx, n_act = dev_empty((NT,), "i32"), dev_empty((NT,), "i32"), dev_empty((1,), "i32")
        compact = dev_empty((S, cap * T, W))
        for t in (flags, idx, n_act, compact):
            t.fill_(-1)
        if static:
            cd.vmajor_select_static(S, N, W, T, cur_d, prev_d, tau, flags, idx, n_act, compact, cap)
        else:
            ws = torch.empty(max(cd.vmajor_select_workspace_bytes(S, N, W, T), 16), dtype=torch.uint8, device="cuda:0")
            cd.vmajor_select(S, N, W, T, cur_d, prev_d, tau, flags, idx, n_act, compact, cap, ws)
        torch.cuda.synchronize()
        outs.append((flags.cpu().numpy(), idx.cpu().numpy(), int(n_act.cpu()[0]), to_host_bits(compact)))
    (f0, i0, n0, c0), (f1, i1, n1, c1) = outs
    assert n0 == n1 == n_changed
    assert np.array_equal(f0, f1) and np.array_equal(i0, i1) and np.array_equal(c0, c1)   # unwritten parts hold the fill on both
    assert np.array_equal(i1[:n1], changed)
    k = min(n1, cap)
    for j in range(k):
        assert np.array_equal(c1[:, j * T:(j + 1) * T], cur[:, changed[j] * T:(changed[j] + 1) * T])


def test_select_static_equals_select_on_two_calls_in_a_row():
    print("select_static: 24 x 9216 x 128, 115 of 576 tiles", flush=True)
    _both(24, 9216, 128, 16, 115, seed=1)            # the 1536 x 1536 image shape, head-parallel
    print("select_static: smaller input on the same library-owned array", flush=True)
    _both(3, 1280, 40, 16, 7, seed=2)                # 80 tiles: the words of the first call beyond them must not matter
    _both(3, 1280, 40, 16, 0, seed=3)                # nothing changed
    _both(1, 4096, 8, 4, 1024, seed=4, cap=5)        # every tile changed, compact smaller than the list


def test_select_static_rejects_more_tiles_than_the_array_holds():
    import ctypes
    from paper_2604_14561_amd import binding as B
    fake = ctypes.c_void_p(0x1000)
    L = B.lib()
    # 65537 tiles of one token
    assert L.cocodiff_vmajor_select_static(1, 65537, 8, 1, fake, fake, 1e-3, None, fake, fake, None, 0, None) == B.ERR_CAPACITY
    assert b"65536" in L.cocodiff_last_error()
    assert L.cocodiff_vmajor_select_static(1, 64, 12, 16, fake, fake, 1e-3, None, fake, fake, None, 0, None) == B.ERR_SHAPE
