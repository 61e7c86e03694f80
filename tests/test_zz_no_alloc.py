"""GPU test of the entry point that allocates nothing (spcfg_inside_static): its workspace is a static device array
inside the library.  Two calls in a row, the second on a smaller batch, each against spcfg_inside on a caller
workspace (fp32 tolerance: the two use different numbers of workgroups, hence different summation splits)."""
import numpy as np
import pytest

from paper_2310_14997_amd import binding as bd
from paper_2310_14997_amd import synth
from parity_util import check_logZ

pytestmark = pytest.mark.gpu


def run_both(d):
    import torch
    wl = bd.Workload(d)
    wl.forward()
    torch.cuda.synchronize()
    ref = wl.logZ.cpu().numpy().astype(np.float64)
    out = torch.full_like(wl.logZ, float("nan"))
    before = torch.cuda.memory_allocated()
    bd.spcfg_inside_static(wl.cfg, wl.log_root, wl.L, wl.R, wl.log_emit, wl.lengths, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return out.cpu().numpy().astype(np.float64), ref


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    from oracle import spcfg_oracle as O
    big = synth.make_inputs("small", seed=4711, pad_value=np.nan, N=200, P=130, B=9,
                            lengths=[30, 12, 2, 25, 18, 7, 30, 3, 21])
    small = synth.make_inputs("tiny", seed=4712, pad_value=np.nan, B=3, lengths=[5, 2, 9])
    for tag, d in (("first call", big), ("second call, smaller batch", small), ("third call, first batch again", big)):
        print("case static scratch:", tag, flush=True)
        got, ref = run_both(d)
        check_logZ(got, ref)
        check_logZ(got, O.inside(d["log_root"], d["L"], d["R"], d["log_emit"], d["lengths"]))


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch
    d = synth.make_inputs("tiny", seed=4713, pad_value=np.nan, B=2, lengths=[4, 3])
    wl = bd.Workload(d)
    cfg = bd.make_config(2048, 2048, 64, 40)
    lens = np.full(64, 40, dtype=np.int32)
    z = torch.zeros(64, device="cuda:0")
    with pytest.raises(bd.SpcfgError) as e:   # refused on the host: the (too small) tensors are never touched
        bd.load()
        import ctypes as C
        rc = bd.load().spcfg_inside_static(C.byref(cfg), wl.log_root.data_ptr(), wl.L.data_ptr(), wl.R.data_ptr(),
                                           wl.log_emit.data_ptr(), lens.ctypes.data, 64, 40, z.data_ptr(), None)
        bd._check(rc)
    assert e.value.code == -7
