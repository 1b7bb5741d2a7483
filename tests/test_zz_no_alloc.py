"""The entry point that allocates nothing (focus_select_compact_noalloc: budget + selection + packing on caller-given
scores and block state, scratch in a fixed device array of the library) against the context-based
focus_select_compact, bit for bit, through the C ABI: two calls in a row, the second with a smaller batch, so that
what the first call left in the shared scratch array is still there when the second runs."""
import numpy as np
import pytest
import torch

import focus_inputs as fi
from test_gpu_parity import DEV, Outs, _pk, install_states

pytestmark = pytest.mark.gpu


def _inputs(r, n, B):
    dI = r.normal(size=(n, B)).astype(np.float32)
    dI[:, ::3] = np.round(dI[:, ::3] * 2) / 2                       # exact ties
    masks = [int(r.integers(0, 1 << B)) for _ in range(n)]
    masks[0], masks[1] = 0, (1 << B) - 1
    sums = [int(r.integers(0, 40)) for _ in range(n)]
    stp = [int(r.integers(0, 9)) for _ in range(n)]
    ko = [int(r.integers(0, B + 1)) for _ in range(n)]
    return dI, masks, sums, stp, ko


@pytest.mark.parametrize("mode,constraints,selection", [(2, 3, 0), (1, 0, 0), (3, 1, 0), (0, 2, 1)])
def test_noalloc_select_compact_equals_context_entry_point_twice(mode, constraints, selection):
    pk, runner = _pk()
    B, n_max = 32, 41
    wl = fi.workload("c1_tiny", block_size=B, batch=n_max, budget_mode=mode, topk=3, keep_ratio=0.2, constraints=constraints,
                     prefill="synthetic", n_layers=2, selection=selection, selection_seed=0xC0FFEE)
    sess = runner.open_session(wl, DEV)
    r = np.random.default_rng(7 + mode)
    for n in (n_max, 13):                                           # the second call is smaller
        dI, masks, sums, stp, ko = _inputs(r, n, B)
        install_states(pk, sess, wl, masks, sums, stp)
        d_dI = torch.from_numpy(dI).to(DEV)
        d_ko = torch.tensor(ko, dtype=torch.int32, device=DEV) if mode == 3 else None
        ref = Outs(pk, wl, n)
        sess.focus.focus_select_compact(n, d_dI, ref.struct, k_override=d_ko)
        g_ref = ref.host()
        got = Outs(pk, wl, n)
        got.t["row_map"].fill_(-7)
        to_i64 = lambda xs: torch.tensor([x - (1 << 64) if x >= (1 << 63) else x for x in xs], dtype=torch.int64, device=DEV)
        pk.focus_select_compact_noalloc(sess.focus.cfg, n, d_dI, to_i64(masks), got.struct,
                                        token_sum=torch.tensor(sums, dtype=torch.int64, device=DEV),
                                        total_steps=torch.tensor(stp, dtype=torch.int32, device=DEV), k_override=d_ko)
        g = got.host()
        T = int(g_ref["cu_seqlens"][n])
        assert np.array_equal(g["K"], g_ref["K"])
        assert np.array_equal(g["keep_bits"], g_ref["keep_bits"])
        assert np.array_equal(g["cu_seqlens"], g_ref["cu_seqlens"])
        assert np.array_equal(g["row_map"][:T], g_ref["row_map"][:T])
        assert np.all(g["row_map"][T:] == -7)                       # nothing written beyond the packed rows
    sess.focus.focus_free()


def test_noalloc_rejects_sizes_beyond_the_scratch_and_missing_arguments():
    pk, runner = _pk()
    wl = fi.workload("c1_tiny", block_size=16, batch=2, budget_mode=2, prefill="synthetic")
    cfg = runner.config_from_workload(wl, 2, 64, 8)
    n = 2
    z = lambda *s, dt: torch.zeros(*s, dtype=dt, device=DEV)
    out = pk.make_step_out(K=z(n, dt=torch.int32), keep_bits=z(n, dt=torch.int64), cu_seqlens=z(n + 1, dt=torch.int32),
                           row_map=z(n * 16, dt=torch.int32))
    dI, mb = z(n, 16, dt=torch.float32), z(n, dt=torch.int64)
    with pytest.raises(pk.FocusError) as e:
        pk.focus_select_compact_noalloc(cfg, pk.FOCUS_NOALLOC_MAX_SEQ + 1, dI, mb, out, token_sum=mb, total_steps=z(n, dt=torch.int32))
    assert e.value.code == pk.FOCUS_EINVAL and "FOCUS_NOALLOC_MAX_SEQ" in str(e.value)
    with pytest.raises(pk.FocusError):                              # dynamic budget without statistics
        pk.focus_select_compact_noalloc(cfg, n, dI, mb, out)
    pk.focus_select_compact_noalloc(cfg, 0, dI, mb, out)             # empty batch: nothing to do
