"""CPU-side checks of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, and its pure host arithmetic (storage sizes, parameter counts, argument
validation that precedes any GPU call) is right."""
import ctypes as C
import os
import re

import pytest

from paper_1801_03138_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ingpu_replay.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_]+)\s*\([^;{]*\)\s*;", text)
    return sorted(set(n for n in names if n.startswith(("replay_", "train_", "rp_", "inram_"))))


def test_header_and_binding_agree():
    declared = _declared_functions()
    assert len(declared) >= 20
    assert declared == sorted(binding.SYMBOLS)


def test_library_exports_every_declared_symbol():
    lib = C.CDLL(binding.LIB_PATH)
    for name in _declared_functions():
        assert hasattr(lib, name), name
    assert b"gfx950" in binding.lib().rp_version()


def test_storage_arithmetic_matches_the_paper(golden_dir):
    """1,000,000 rows of 57 four-byte values (Methods); rows are stored padded to 256 bytes."""
    cfg = binding.ReplayConfig(1_000_000, 27, binding.RP_F32, binding.RP_PAIR, 2000, 50_000, 0)
    assert (2 * 27 + 3) * 4 == 228 <= binding.row_bytes(cfg) == 256
    need = binding.storage_bytes(cfg)
    assert 1_000_000 * 256 <= need <= 1_000_000 * 256 + (1 << 20)
    # pixel states, one per experience (Discussion): 84*84*4 bytes plus 9 bytes of scalars
    big = binding.ReplayConfig(200_000, 84 * 84 * 4, binding.RP_U8, binding.RP_CHAIN, 64, 0, 0)
    assert 28224 + 9 <= binding.row_bytes(big) <= 28224 + 128 + 9
    assert 200_000 * 28224 <= binding.storage_bytes(big) <= 200_000 * (28224 + 128 + 9) + (1 << 22)
    bf = binding.ReplayConfig(4_000_000, 27, binding.RP_BF16, binding.RP_PAIR, 64, 0, 0)
    assert binding.row_bytes(bf) == 128


@pytest.mark.parametrize("cfg", [
    (0, 27, 0, 0, 1), (2**32, 27, 0, 0, 1), (10, 0, 0, 0, 1), (10, 27, 3, 0, 1), (10, 27, 0, 2, 1),
    (10, 27, 0, 0, 0), (10, 20000, 0, 0, 1)])
def test_invalid_replay_configurations_have_no_size(cfg):
    c = binding.ReplayConfig(cfg[0], cfg[1], cfg[2], cfg[3], cfg[4], 0, 0)
    assert binding.storage_bytes(c) == 0 and binding.row_bytes(c) == 0


def test_param_count_and_workspace():
    lib = binding.lib()
    cfg = binding.TrainConfig(27, 256, 30, 128, binding.RP_F32, 0, 1, 1, 1e-4, 0.99, 0.9, 0.999,
                              1e-8, 1)
    assert lib.train_param_count(C.byref(cfg)) == 27 * 256 + 256 + 256 * 256 + 256 + 256 * 30 + 30 == 80670
    assert lib.train_workspace_bytes(C.byref(cfg)) > 4 * 4 * 80670
    wide = binding.TrainConfig(27, 1024, 30, 4096, binding.RP_BF16, 0, 1, 64, 1e-4, 0.99, 0.9,
                               0.999, 1e-8, 1)
    assert lib.train_param_count(C.byref(wide)) == 1_109_022
    bad = binding.TrainConfig(27, 100, 30, 128, binding.RP_F32, 0, 1, 1, 1e-4, 0.99, 0.9, 0.999,
                              1e-8, 1)
    assert lib.train_param_count(C.byref(bad)) == 0 and lib.train_workspace_bytes(C.byref(bad)) == 0


def test_null_arguments_are_rejected_before_any_gpu_call():
    lib = binding.lib()
    assert lib.replay_create(None, None, 0, None) == binding.RP_EINVAL
    assert b"null" in lib.rp_last_error()
    assert lib.replay_append(None, 1, None, None, None, None, None, 0, None) == binding.RP_EINVAL
    assert lib.replay_sample_gather(None, 0, 1, None, None, None, None, None, None, None) == binding.RP_EINVAL
    assert lib.train_step(None, None, None, None, None, None, 0, None) == binding.RP_EINVAL
    assert lib.train_create(None, None, None, 0, None, None) == binding.RP_EINVAL
    assert lib.replay_destroy(None) == 0 and lib.train_destroy(None) == 0
    assert lib.train_step_batch(None, None, None, None, None, None, None) == binding.RP_EINVAL
    assert lib.inram_create(10, 4, 0, 0, 2, None, 0, None) == binding.RP_EINVAL
    assert lib.inram_train_step(None, None, None) == binding.RP_EINVAL
    assert lib.inram_destroy(None) == 0
    assert lib.inram_device_bytes(27, 128) >= 128 * (2 * 27 * 4 + 9) and lib.inram_device_bytes(0, 1) == 0
