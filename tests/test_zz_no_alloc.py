"""The allocation-free bounds entry point (csv_bounds_static) against csv_bounds, through the C ABI.

Two calls in a row on one GPU, the second with a smaller input: the static scratch array keeps the first call's
partial sums, which the second call must not see."""
import numpy as np
import pytest

import synth

from ._harness import Case, log

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_static_bounds_match_the_workspace_entry_point_bit_for_bit():
    r = synth.small_recipe("static", V=3001, d=520, C=37, B=40, steps=2, h_mode="mix", iso_frac=0.2)
    case = Case(r, seed=61)
    csv = case.csv
    h = case.hidden()
    dh = csv.bits_to_device(h)
    # first call: 40 sequences (batched product, partial sums in the static array); second: 12 sequences of another
    # step (fewer partial sums, the rest of the array still holds the first call's); third: 3 sequences (no scratch)
    for tag, hb in (("B=40", dh[0]), ("B=12", dh[1][5:17].contiguous()), ("B=3", dh[0][:3].contiguous()), ("B=40 again", dh[1])):
        B = hb.shape[0]
        log(f"csv_bounds_static {tag}")
        want_U, want_hn = csv.csv_bounds(case.ws, case.gidx, hb)
        U = torch.full((B, case.gidx.C), float("nan"), dtype=torch.float32, device="cuda")
        hn = torch.full((B,), float("nan"), dtype=torch.float32, device="cuda")
        csv.csv_bounds_static(case.gidx, hb, U, hn)
        torch.cuda.synchronize()
        assert np.array_equal(U.cpu().numpy().view(np.uint32), want_U.cpu().numpy().view(np.uint32)), tag
        assert np.array_equal(hn.cpu().numpy().view(np.uint32), want_hn.cpu().numpy().view(np.uint32)), tag
    case.close()


def test_static_bounds_reject_what_the_scratch_cannot_hold():
    import paper_2511_21702_amd as csv
    V, d, C = 8200, 256, 8192
    W = torch.zeros((V, d), dtype=torch.int16, device="cuda")
    n = np.ones(C, np.int32)
    n[0] += V - C
    idx = csv.csv_index_from_arrays(W, None, np.zeros((C, d), np.float32), np.ones(C, np.float32), np.zeros(C, np.float32), n,
                                    np.arange(V, dtype=np.int32))
    h = torch.zeros((256, d), dtype=torch.int16, device="cuda")
    U = torch.zeros((256, C), dtype=torch.float32, device="cuda")
    hn = torch.zeros(256, dtype=torch.float32, device="cuda")
    with pytest.raises(csv.CsvError) as e:
        csv.csv_bounds_static(idx, h, U, hn)                  # 2 K slices x 256 x 8192 floats = 16 MiB > 8 MiB
    assert e.value.code == -4 and "static scratch" in str(e.value)
    csv.csv_bounds_static(idx, h[:4], U[:4], hn[:4])          # up to 4 sequences need no scratch at all
    csv.csv_bounds_static(idx, h[:100], U[:100], hn[:100])    # 2 x 100 x 8192 floats fit
    torch.cuda.synchronize()
    assert np.all(U[:100].cpu().numpy() == 0.0)               # h = 0: every bound is the bias maximum, 0
    idx.free()
