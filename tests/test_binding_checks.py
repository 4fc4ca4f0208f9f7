"""The Python binding refuses device arrays that do not fit what the kernels will read or write
(the C interface carries no lengths), before anything is launched.  Runs without a GPU: the checks
are plain functions over tensor metadata."""
import numpy as np
import pytest
import torch

from paper_1801_03138_amd import binding as B

CPU = torch.device("cpu")


def _cfg(D=5, dtype=B.RP_F32, layout=B.RP_PAIR):
    return B.ReplayConfig(64, D, dtype, layout, 16, 0, 0, B.RP_WITH_REPLACEMENT, 0)


def _rows(n, D, state=torch.float32):
    return dict(s=torch.zeros(n, D, dtype=state), s_next=torch.zeros(n, D, dtype=state),
                a=torch.zeros(n, dtype=torch.int32), r=torch.zeros(n, dtype=torch.float32),
                term=torch.zeros(n, dtype=torch.uint8))


def test_well_formed_device_experiences_pass():
    r = _rows(7, 5)
    B.check_device_experiences(_cfg(), CPU, 7, r["s"], r["s_next"], r["a"], r["r"], r["term"], "t")
    # bf16 states may travel as bfloat16 or as their 16-bit patterns; CHAIN replays ignore s_next
    for st in (torch.bfloat16, torch.int16):
        r = _rows(3, 5, st)
        B.check_device_experiences(_cfg(dtype=B.RP_BF16), CPU, 3, r["s"], r["s_next"], r["a"], r["r"],
                                   r["term"], "t")
    r = _rows(3, 5, torch.uint8)
    B.check_device_experiences(_cfg(dtype=B.RP_U8, layout=B.RP_CHAIN), CPU, 3, r["s"], None, r["a"], r["r"],
                               r["term"], "t")


@pytest.mark.parametrize("field,bad,why", [
    ("s", lambda r: r["s"][:6], "short"),
    ("s_next", lambda r: r["s_next"][:, :4], "strided and short"),
    ("s", lambda r: r["s"].double(), "wrong dtype"),
    ("a", lambda r: r["a"].long(), "wrong dtype"),
    ("a", lambda r: r["a"][:3], "short"),
    ("r", lambda r: r["r"].half(), "wrong dtype"),
    ("r", lambda r: torch.zeros(14)[::2], "strided"),
    ("term", lambda r: r["term"].int(), "wrong dtype"),
    ("term", lambda r: r["term"].numpy(), "not a tensor"),
    ("s_next", lambda r: None, "missing"),
])
def test_malformed_device_experiences_are_refused(field, bad, why):
    r = _rows(7, 5)
    r[field] = bad(r)
    with pytest.raises(ValueError):
        B.check_device_experiences(_cfg(), CPU, 7, r["s"], r["s_next"], r["a"], r["r"], r["term"], why)


def test_tensor_on_another_device_is_refused():
    r = _rows(7, 5)
    with pytest.raises(ValueError, match="is on cpu"):
        B.check_device_experiences(_cfg(), torch.device("cuda:0"), 7, r["s"], r["s_next"], r["a"], r["r"],
                                   r["term"], "t")


def test_sample_outputs_are_checked_against_the_batch():
    cfg, batch = _cfg(), 9
    good = lambda: (torch.zeros(batch, 5), torch.zeros(batch, 5), torch.zeros(batch, dtype=torch.int32),
                    torch.zeros(batch), torch.zeros(batch, dtype=torch.uint8),
                    torch.zeros(batch, dtype=torch.int32))
    B.check_batch_out(cfg, CPU, batch, good(), "t")
    B.check_batch_out(cfg, CPU, batch, good()[:5] + (None,), "t")         # idx is optional
    for k, bad in ((0, torch.zeros(batch - 1, 5)), (1, torch.zeros(batch, 5, dtype=torch.bfloat16)),
                   (2, torch.zeros(batch, dtype=torch.int64)), (3, torch.zeros(2 * batch)[::2]),
                   (4, torch.zeros(batch, dtype=torch.bool)), (5, torch.zeros(batch + 1, dtype=torch.int32))):
        out = list(good())
        out[k] = bad
        with pytest.raises(ValueError):
            B.check_batch_out(cfg, CPU, batch, tuple(out), "t")
    with pytest.raises(ValueError):
        B.check_batch_out(cfg, CPU, batch, good()[:4], "t")
    # uint8 states come out as float32, bf16 states as bf16
    u8 = list(good())
    B.check_batch_out(_cfg(dtype=B.RP_U8, layout=B.RP_CHAIN), CPU, batch, tuple(u8), "t")
    bf = list(good())
    bf[0], bf[1] = bf[0].bfloat16(), bf[1].bfloat16()
    B.check_batch_out(_cfg(dtype=B.RP_BF16), CPU, batch, tuple(bf), "t")
    with pytest.raises(ValueError):
        B.check_batch_out(_cfg(dtype=B.RP_BF16), CPU, batch, good(), "t")


def test_host_arrays_are_checked_for_length():
    D, n = 5, 4
    ok = [np.zeros((n, D), np.float32), np.zeros((n, D), np.float32), np.zeros(n, np.int32),
          np.zeros(n, np.float32), np.zeros(n, np.uint8)]
    B.check_host_experiences(_cfg(), n, *ok, "t")
    for k in range(5):
        bad = list(ok)
        bad[k] = bad[k][:-1]
        with pytest.raises(ValueError):
            B.check_host_experiences(_cfg(), n, *bad, "t")
    B.check_host_experiences(_cfg(layout=B.RP_CHAIN), n, ok[0], None, ok[2], ok[3], ok[4], "t")
