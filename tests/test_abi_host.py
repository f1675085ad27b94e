"""Host-side checks that need no GPU: the C-ABI library loads, exports every
symbol the header declares, and its host-only planning logic is right."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "cdgrab.h")


@pytest.fixture(scope="module")
def p():
    import paper_2302_00845_amd as pkg
    if not os.path.exists(pkg.library_path()):
        from paper_2302_00845_amd import build
        build.build_library(verbose=False)
    return pkg


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(cdgrab_[a-z0-9_]+)\s*\(", text))
    names -= {"cdgrab_gen_fn"}
    return sorted(names)


def test_header_declares_the_expected_calls():
    names = declared_symbols()
    for required in ("cdgrab_pergrad", "cdgrab_balance_epoch", "cdgrab_reorder", "cdgrab_create",
                     "cdgrab_destroy", "cdgrab_last_error", "cdgrab_plan_epoch", "cdgrab_get_timing",
                     "cdgrab_herding_bound", "cdgrab_train_epoch_softmax", "cdgrab_train_softmax",
                     "cdgrab_balance_epoch_independent",
                     "cdgrab_balance_epoch_stale_mean", "cdgrab_balance_epoch_randomized"):
        assert required in names


def test_library_exports_every_declared_symbol(p):
    lib = ctypes.CDLL(p.library_path())
    for name in declared_symbols():
        assert hasattr(lib, name), "libcdgrab.so does not export %s" % name


def test_missing_library_fails_loudly(p, monkeypatch):
    from paper_2302_00845_amd import cdgrab
    monkeypatch.setattr(cdgrab, "_lib", None)
    monkeypatch.setattr(cdgrab, "_LIB_PATH", "/nonexistent/libcdgrab.so")
    with pytest.raises(FileNotFoundError):
        cdgrab.load_library()


def test_plan_epoch_headline_shapes(p):
    c4 = p.cdgrab_plan_epoch(32, 512, 11_200_000, streamed=True)
    assert c4["pairs"] == 8192 and c4["block_pairs"] == 32 and c4["blocks"] == 256
    assert c4["vector_width"] == 4
    assert c4["staging_bytes"] == 32 * 2 * 11_200_000 * 4 and c4["fused_apply"] == 0
    assert c4["bytes_per_example"] == 8 * 11_200_000 + 12 * 11_200_000 / 32
    c3 = p.cdgrab_plan_epoch(32, 1024, 1 << 20, streamed=True)
    assert c3["fused_apply"] == 1 and c3["staging_bytes"] == 2 * 32 * 2 * (1 << 20) * 4
    assert c3["bytes_per_example"] == 8 * (1 << 20) + 8 * (1 << 20) / 32
    c2 = p.cdgrab_plan_epoch(16, 3750, 7850)
    assert c2["pairs"] == 30000 and c2["block_pairs"] == 64 and c2["blocks"] == 469 and c2["vector_width"] == 2
    assert c2["staging_bytes"] == 0
    # short dense rows: Gram matrices ahead, rows read three times; that form applies a block
    # inside its own launch, so it is not reported as the fused dot/Gram launch
    assert c2["gram_ahead"] == 1 and c2["bytes_per_example"] == 12 * 7850 + 8 * 7850 / 64
    assert c2["fused_apply"] == 0
    # its workspace counts the buffers of that form: reduced Gram tiles of 469 blocks (+1 carried
    # over), two blocks' per-workgroup dots, the row maps, and partials for all blocks' workgroups
    part = 10 * 256 + 64
    groups = -(-4 * 256 // 469)
    assert c2["workspace_bytes"] >= 469 * groups * part * 8 + 470 * part * 8 + 2 * 123 * 64 * 8
    # long streamed rows: running sum + partials of 512 workgroups + one staging block
    assert c4["workspace_bytes"] >= 11_200_000 * 8 + 512 * (3 * 256 + 32) * 8 + c4["staging_bytes"]
    assert c4["workspace_bytes"] < 11_200_128 * 8 + 512 * (3 * 256 + 32) * 8 + c4["staging_bytes"] + (1 << 20)
    assert c4["gram_ahead"] == 0 and c3["gram_ahead"] == 0
    assert p.cdgrab_plan_epoch(16, 3750, 7850, streamed=True)["gram_ahead"] == 0
    assert p.cdgrab_plan_epoch(4, 64, 100_000)["gram_ahead"] == 0
    odd = p.cdgrab_plan_epoch(3, 4, 1001, base_align=4)
    assert odd["vector_width"] == 1 and odd["block_pairs"] == 16 and odd["blocks"] == 1
    assert p.cdgrab_plan_epoch(1, 2, 1)["pass1_groups"] == 1
    assert p.cdgrab_plan_epoch(1, 66, 8, block_pairs=16)["blocks"] == 3


@pytest.mark.parametrize("args", [(0, 4, 4), (2, 3, 4), (2, 0, 4), (2, 4, 0), (2, -2, 4)])
def test_plan_epoch_rejects_bad_sizes(p, args):
    with pytest.raises(p.CdgrabError) as ei:
        p.cdgrab_plan_epoch(*args)
    assert ei.value.code == -1


def test_plan_epoch_rejects_bad_block_and_overflow(p):
    with pytest.raises(p.CdgrabError):
        p.cdgrab_plan_epoch(2, 4, 4, block_pairs=24)
    with pytest.raises(p.CdgrabError):
        p.cdgrab_plan_epoch(2 ** 31, 2 ** 31, 2 ** 31)


def test_null_handle_is_an_error_not_a_crash(p):
    lib = p.load_library()
    assert lib.cdgrab_balance_epoch(None, 1, 2, 1, None, None, None, None, None, None, None, None, None) == -1
    assert lib.cdgrab_reorder(None, 1, 1, None, None, None) == -1
    assert lib.cdgrab_pergrad(None, 1, 1, 1, None, None, None, None) == -1
    assert lib.cdgrab_destroy(None) == 0
