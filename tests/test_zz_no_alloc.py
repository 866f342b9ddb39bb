"""rtp_topp_select_noalloc (scratch built into the library, nothing allocated) against rtp_topp_select with a
caller workspace: same kernels, so every output must be bit-identical -- on two calls in a row, the second with a
smaller input (the built-in buffer keeps the first call's contents)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2605_16928_amd import rtp
from gpu_util import DEV, i32

pytestmark = pytest.mark.gpu


def _rows(rng, R, n_max, spread):
    lens = [n_max] + [int(x) for x in rng.integers(1, n_max + 1, size=R - 1)]
    stride = (n_max + 3) // 4 * 4
    sc = torch.full((R, stride), float("nan"), dtype=torch.float32)
    for r, n in enumerate(lens):
        s = rng.standard_normal(n) * spread
        s[rng.integers(0, n, size=min(n, 20))] += 6.0
        sc[r, :n] = torch.from_numpy(s.astype(np.float32))
    p = torch.tensor(rng.choice([0.5, 0.8, 0.9, 0.99, 1.0], size=R), dtype=torch.float32)
    return sc.to(DEV), i32(lens), p.to(DEV), stride


def _outputs(R, stride):
    return (torch.full((R, stride), -1, dtype=torch.int32, device=DEV), torch.full((R,), -9, dtype=torch.int32, device=DEV),
            torch.zeros(R, device=DEV), torch.zeros(R, device=DEV))


def test_topp_select_noalloc_matches_the_workspace_form():
    print("[case] top-p without a caller workspace", flush=True)
    lib = rtp.lib()
    vp = C.c_void_p
    rng = np.random.default_rng(31)
    for (R, n_max, spread) in ((12, 70000, 1.0), (3, 9001, 0.3)):        # the second call is the smaller one
        sc, row_len, p, stride = _rows(rng, R, n_max, spread)
        sel_a, cnt_a, tau_a, mass_a = _outputs(R, stride)
        sel_b, cnt_b, tau_b, mass_b = _outputs(R, stride)
        ws = torch.empty(rtp.rtp_topp_workspace_bytes(R, n_max), dtype=torch.uint8, device=DEV)
        rtp.rtp_topp_select(sc, stride, row_len, p, R, n_max, sel_a, stride, cnt_a, tau_a, mass_a, ws)
        # the new entry point, straight through the C ABI
        rc = lib.rtp_topp_select_noalloc(vp(sc.data_ptr()), stride, vp(row_len.data_ptr()), vp(p.data_ptr()), R, n_max,
                                         vp(sel_b.data_ptr()), stride, vp(cnt_b.data_ptr()), vp(tau_b.data_ptr()),
                                         vp(mass_b.data_ptr()), vp(torch.cuda.current_stream().cuda_stream))
        assert rc == rtp.RTP_OK, lib.rtp_last_error()
        torch.cuda.synchronize()
        assert torch.equal(cnt_a, cnt_b) and int(cnt_a.min()) > 0
        assert torch.equal(tau_a, tau_b) and torch.equal(mass_a, mass_b)
        for r in range(R):
            c = int(cnt_a[r])
            assert torch.equal(sel_a[r, :c], sel_b[r, :c]), f"row {r}"
    # beyond the built-in buffer: refused, nothing enqueued
    rc = lib.rtp_topp_select_noalloc(vp(sc.data_ptr()), 1 << 20, vp(row_len.data_ptr()), vp(p.data_ptr()), 512, 1 << 20,
                                     vp(sel_b.data_ptr()), 1 << 20, vp(cnt_b.data_ptr()), None, None, None)
    assert rc == rtp.RTP_ERR_WORKSPACE and b"built-in" in lib.rtp_last_error()
