"""The entry point that allocates nothing (static device scratch) against the entry point it is a variant of:
two calls in a row through the C ABI, the second on a smaller input (needs an MI355X)."""
import numpy as np
import pytest

import tsdp_inputs as ti
from tests.helpers import gpu_side, to_dev

pytestmark = pytest.mark.gpu


def test_distill_loss_noalloc_matches_the_allocating_entry_point():
    import torch
    from paper_2512_15773_amd import TsdpError
    wl = ti.small_variant(ti.C3, B=40, base=ti.NetShape(1, 256, 4), draft=ti.NetShape(1, 128, 4))
    wb, wd = ti.make_weights(wl, "base", b_std=0.02), ti.make_weights(wl, "draft", b_std=0.02)
    cond, x = ti.make_cond(wl, 40), ti.make_latents(wl, 40)
    rng = np.random.default_rng(21)
    t0 = rng.integers(0, 100, 40).astype(np.int32); K = rng.integers(1, 17, 40).astype(np.int32)
    s = np.ones(40, np.float32)
    for clip in (None, 1.5):
        ctx = gpu_side(wl, wb, wd, cond, clip=clip)
        rows = ctx.alloc_rows(40)
        ctx.tsdp_draft(to_dev(x), to_dev(t0), to_dev(K), to_dev(s), None, rows)
        ctx.tsdp_verify(40, rows)
        R = int(rows["row_ptr"].cpu().numpy()[-1])
        assert R > 300                                             # several workgroups of partial sums and a ragged tail
        loss = torch.zeros(3, dtype=torch.float64, device="cuda")
        for n in (R, 37):                                          # the second call is smaller: stale partial sums stay behind it
            want = ctx.tsdp_distill_loss(n, rows, 0.7, 0.3).cpu().numpy()
            loss.fill_(-1.0)
            ctx.tsdp_distill_loss_noalloc(n, rows, 0.7, 0.3, loss)
            got = loss.cpu().numpy()
            assert got.tobytes() == want.tobytes(), (n, got, want)
            assert got[0] > 0 and got[1] > 0
        ctx.tsdp_distill_loss_noalloc(0, rows, 0.7, 0.3, loss)     # empty input: zeros, no launch over rows
        assert loss.cpu().numpy().tolist() == [0.0, 0.0, 0.0]
        ctx.close()
    # beyond the static scratch the call is refused with a clear error
    big = ti.small_variant(wl, B=4200)
    ctx = gpu_side(big, wb, wd, ti.make_cond(big, 4200), B_max=4200)
    rows = {k: torch.zeros(1, device="cuda", dtype=torch.int32 if k == "row_t" else torch.float32)
            for k in ("row_t", "states", "eps_p", "eps_q")}
    with pytest.raises(TsdpError) as e:
        ctx.tsdp_distill_loss_noalloc(65537, rows, 1.0, 1.0, torch.zeros(3, dtype=torch.float64, device="cuda"))
    assert e.value.code == -2 and "65536" in str(e.value)
    ctx.close()
