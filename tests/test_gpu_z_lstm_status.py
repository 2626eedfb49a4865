"""GPU: status word and host-forced give-up path of the LSTM recurrence that runs in one launch."""
import numpy as np
import pytest
import torch

from paper_2203_05705_amd import binding as ard
from util import from_vals, stored

pytestmark = pytest.mark.gpu


def test_one_launch_recurrence_status_and_give_up_path():
    """The forward recurrence in one launch leaves its status word at 0; with a negative wait bound set from
    the host every workgroup's first wait fails: they give up, leave normally and set the word; the next call
    is unaffected."""
    import os
    T, B, I, H, dp = 12, 128, 256, 1024, 2
    dt = ard.BF16
    pat = ard.Pattern.row(dp, 1)
    off = ard.lstm_status_offset(dt, T, B, I, H, pat)
    assert off is not None and ard.lstm_status_offset(ard.F32, T, B, I, H, pat) is None
    rng = np.random.default_rng(5)
    x = from_vals(stored(rng.standard_normal((T, B, I)), "bf16"), "bf16")
    W = from_vals(stored(rng.uniform(-0.05, 0.05, (4 * H, I + H)), "bf16"), "bf16")
    ws = torch.empty(ard.lstm_workspace_bytes(dt, T, B, I, H, pat), dtype=torch.uint8, device="cuda")
    status = lambda: int(ws[off:off + 4].view(torch.int32).item())
    h0, c0, g0 = ard.lstm_fwd(x, W, pat, ws=ws)
    torch.cuda.synchronize()
    assert status() == 0, "a complete call left the status word set"
    assert bool(torch.isfinite(h0.float()).all()), "h of a complete call holds unwritten entries"
    os.environ["ARD_LSTM_SPIN_LIMIT"] = "-1"
    try:
        print("forcing the give-up path (negative spin limit)", flush=True)
        ard.lstm_fwd(x, W, pat, ws=ws)
        torch.cuda.synchronize()          # every workgroup left on its own
        assert status() == 1, "no workgroup gave up although the wait bound was negative"
    finally:
        del os.environ["ARD_LSTM_SPIN_LIMIT"]
    h1, c1, g1 = ard.lstm_fwd(x, W, pat, ws=ws)
    torch.cuda.synchronize()
    assert status() == 0, "the call after a given-up one left the status word set"
    for name, a, b in (("h", h1, h0), ("c", c1, c0), ("gates", g1, g0)):
        assert torch.equal(a, b), f"{name} differs between two identical calls: {int((a != b).sum())} entries, " \
                                  f"max |d| {float((a.float() - b.float()).abs().max()):.3e}"


def test_backward_recurrence_give_up_path():
    """The backward recurrence in one launch shares the status word and the bounded wait: forced to give up it
    leaves normally with the word set, and the next call gives the results of an undisturbed one."""
    import os
    T, B, I, H, dp = 10, 128, 128, 1024, 2
    dt = ard.BF16
    pat = ard.Pattern.row(dp, 2)
    off = ard.lstm_status_offset(dt, T, B, I, H, pat)
    assert off is not None
    rng = np.random.default_rng(6)
    x = from_vals(stored(rng.standard_normal((T, B, I)), "bf16"), "bf16")
    W = from_vals(stored(rng.uniform(-0.05, 0.05, (4 * H, I + H)), "bf16"), "bf16")
    dh = from_vals(stored(rng.standard_normal((T, B, H)), "bf16"), "bf16")
    ws = torch.empty(ard.lstm_workspace_bytes(dt, T, B, I, H, pat), dtype=torch.uint8, device="cuda")
    status = lambda: int(ws[off:off + 4].view(torch.int32).item())
    h, c, g = ard.lstm_fwd(x, W, pat, ws=ws)
    dx0, dW0 = ard.lstm_bwd(x, W, pat, h, c, g, dh, ws=ws)
    torch.cuda.synchronize()
    assert status() == 0, "a complete backward call left the status word set"
    os.environ["ARD_LSTM_SPIN_LIMIT"] = "-1"
    try:
        print("forcing the give-up path of the backward recurrence (negative spin limit)", flush=True)
        ard.lstm_bwd(x, W, pat, h, c, g, dh, ws=ws)
        torch.cuda.synchronize()          # every workgroup left on its own
        assert status() == 1, "no workgroup gave up although the wait bound was negative"
    finally:
        del os.environ["ARD_LSTM_SPIN_LIMIT"]
    dx1, dW1 = ard.lstm_bwd(x, W, pat, h, c, g, dh, ws=ws)
    torch.cuda.synchronize()
    assert status() == 0, "the call after a given-up one left the status word set"
    assert torch.equal(dx1, dx0) and torch.equal(dW1, dW0), "results differ after a given-up call"
