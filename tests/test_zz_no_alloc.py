"""ps_anticipate_static (the entry point that allocates nothing: its partial curves live in a fixed array inside
the library's device image) against ps_anticipate on the same inputs: bit-equal maps, two calls in a row, the
second on a smaller input, so that whatever the first call left in the shared array is there to disturb it."""
import numpy as np
import pytest
import torch

from paper_2504_03702_amd import binding as ps
from paper_2504_03702_amd import workloads as wl
from tests.gpu_util import run_anticipate

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_static(inp, load=None, overflow=None):
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int32)).to(DEV)
    load_t = torch.zeros(inp.n_inst * inp.horizon, dtype=torch.int32, device=DEV) if load is None \
        else torch.from_numpy(np.ascontiguousarray(load, np.int32).reshape(-1)).to(DEV)
    ovf_t = torch.zeros(inp.n_inst, dtype=torch.int64, device=DEV) if overflow is None \
        else torch.from_numpy(np.ascontiguousarray(overflow, np.int64)).to(DEV)
    rate = None if inp.rate is None else t(inp.rate)
    st = ps.new_status(DEV)
    ps.ps_anticipate_static(t(inp.pred_tokens), t(inp.instance_id), t(inp.arrival_bucket), rate, inp.n_inst,
                            inp.horizon, load_t, ovf_t, st)
    flags, bad = ps.ps_status_read(st)
    return load_t.cpu().numpy().reshape(inp.n_inst, inp.horizon), ovf_t.cpu().numpy(), flags, bad


def test_two_calls_in_a_row_match_the_workspace_entry_point():
    big = wl.make_anticipator_inputs("production", seed=11, n=150_000)     # 10 parts of the record stream
    small = wl.make_anticipator_inputs("production", seed=12, n=4096)      # one part: the production batch
    print("ps_anticipate_static production n=150000 then n=4096", flush=True)
    for inp in (big, small):
        want_load, want_ovf, want_flags, _ = run_anticipate(inp)
        got_load, got_ovf, flags, _ = run_static(inp)
        assert flags == want_flags == 0
        assert np.array_equal(got_load, want_load) and np.array_equal(got_ovf, want_ovf)
        per_inst = np.bincount(inp.instance_id, weights=inp.pred_tokens, minlength=inp.n_inst).astype(np.int64)
        assert np.array_equal(got_load.sum(axis=1, dtype=np.int64) + got_ovf, per_inst)
    # a third, smaller still and of another shape (no rate: spread to the end of the horizon), accumulated
    # into a map that already holds values
    tiny = wl.make_anticipator_inputs("tiny", seed=13, n=16)
    rng = np.random.default_rng(0)
    load0 = rng.integers(-50, 50, (tiny.n_inst, tiny.horizon)).astype(np.int32)
    want_load, want_ovf, _, _ = run_anticipate(tiny, load0)
    got_load, got_ovf, flags, _ = run_static(tiny, load0)
    assert flags == 0 and np.array_equal(got_load, want_load) and np.array_equal(got_ovf, want_ovf)


def test_faulty_records_and_limits():
    inp = wl.make_anticipator_inputs("small", seed=4, n=500)
    inp.pred_tokens[17] = -5
    inp.arrival_bucket[0] = -2
    want_load, want_ovf, want_flags, want_bad = run_anticipate(inp)
    got_load, got_ovf, flags, bad = run_static(inp)
    assert flags == want_flags == ps.PS_ST_BAD_RECORD and bad == want_bad == 0
    assert np.array_equal(got_load, want_load) and np.array_equal(got_ovf, want_ovf)
    # beyond the array: refused on the host, nothing is launched
    z = torch.zeros(4, dtype=torch.int32, device=DEV)
    assert ps.ps_anticipate_workspace_bytes(300_000, 256, 600) > ps.PS_ANTICIPATE_STATIC_BYTES
    lib = ps.load_library()
    rc = lib.ps_anticipate_static(z.data_ptr(), z.data_ptr(), z.data_ptr(), None, 300_000, 256, 600, z.data_ptr(),
                                  None, None, None)
    assert rc == -5                                                           # PS_EWORKSPACE
    rc = lib.ps_anticipate_static(z.data_ptr(), z.data_ptr(), z.data_ptr(), None, 4, 1, 70_000, z.data_ptr(),
                                  None, None, None)
    assert rc == -6                                                           # PS_EUNSUPPORTED: horizon
    ps.ps_anticipate_static(z[:0], z[:0], z[:0], None, 2, 2, z, None)       # no records: nothing to do
