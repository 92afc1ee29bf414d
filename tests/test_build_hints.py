"""The fused update keeps a leading part of theta, v, m in the memory-side cache by giving the leading blocks a
path without non-temporal hints.  The paths differ only in hints, which an optimiser is free to merge (dropping the
hints, and with them the mechanism, without any functional symptom).  This test compiles the kernels' source to
gfx950 assembly with the library's own flags and counts the hinted and plain 128-bit accesses per kernel."""
import os
import re
import subprocess

import pytest

from paper_1909_10802_amd import build as ga_build

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def assembly(source, tmp_path):
    out = str(tmp_path / (source + ".s"))
    subprocess.check_call([HIPCC, *ga_build.HIPCC_FLAGS, "-S", "--cuda-device-only", "-x", "hip",
                           os.path.join(ga_build.CSRC, source), "-o", out], stderr=subprocess.DEVNULL)
    return open(out).read()


def kernel_text(asm, mangled_part):
    m = re.search(r"^(_ZN2ga\S*%s\S*):.*?\n(.*?)\.end_amdhsa_kernel" % re.escape(mangled_part), asm, flags=re.S | re.M)
    assert m, mangled_part
    return m.group(2)


def counts(text):
    loads = re.findall(r"global_load_dwordx4 .*", text)
    stores = re.findall(r"global_store_dwordx4 .*", text)
    hinted = lambda xs: sum(1 for x in xs if re.search(r"\bnt\b", x))
    return hinted(loads), len(loads) - hinted(loads), hinted(stores), len(stores) - hinted(stores)


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_cache_hint_paths_survive_the_compiler(tmp_path):
    asm = assembly("ga_apply.hip", tmp_path)
    # apply_kernel<GA, float g, keep m, snapshot, aligned, U>: loads theta, v, m, snapshot, g; stores theta, v, m, snapshot.
    # Paths: all streamed | theta kept | theta, v kept | theta, v, m kept.
    for U in (1,):
        text = kernel_text(asm, "12apply_kernelILi3ELi0ELb1ELb1ELb1ELi%dEE" % U)
        for name in ("all streamed", "theta kept", "theta and v kept", "theta, v and m kept"):
            assert "; %s begin" % name in text and "; %s end" % name in text
        assert counts(text) == ((5 + 4 + 3 + 2) * U, (0 + 1 + 2 + 3) * U, (4 + 3 + 2 + 1) * U, (0 + 1 + 2 + 3) * U)
    # ASGD without Gap tracking: theta, v, g; no m, no snapshot: three paths
    text = kernel_text(asm, "12apply_kernelILi0ELi0ELb0ELb0ELb1ELi1EE")
    assert counts(text) == (3 + 2 + 1, 0 + 1 + 2, 2 + 1 + 0, 0 + 1 + 2)
    # family_apply_kernel<DANA, GA, float g, keep m, snapshot, aligned, 1>: loads theta, x, y, m, snapshot, g
    text = kernel_text(asm, "19family_apply_kernelILi1ELi3ELi0ELb1ELb1ELb1ELi1EE")
    assert counts(text) == (6 + 5 + 4, 0 + 1 + 2, 5 + 4 + 3, 0 + 1 + 2)


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_layerwise_hint_paths_survive_the_compiler(tmp_path):
    asm = assembly("ga_layerwise.hip", tmp_path)
    # layer_apply_kernel<float g, aligned, heavy ball, LOOK>: two groups per thread; loads theta, v, m, g, next snapshot
    text = kernel_text(asm, "18layer_apply_kernelILi0ELb1ELb0ELb1EE")
    hinted_loads, plain_loads, hinted_stores, plain_stores = counts(text)
    assert (hinted_loads, plain_loads) == ((5 + 4 + 3) * 2, (0 + 1 + 2) * 2)
    assert hinted_stores == (4 + 3 + 2) * 2 and plain_stores == (0 + 1 + 2) * 2 + 1     # + the chunk's partial sums


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_gap_statistics_hint_paths_survive_the_compiler(tmp_path):
    asm = assembly("ga_aux.hip", tmp_path)
    # diag_kernel: two groups in flight per thread; loads theta, snapshot, m.  Paths: theta kept | all streamed.
    text = kernel_text(asm, "11diag_kernel")
    for name in ("theta kept", "all streamed"):
        assert "; %s begin" % name in text and "; %s end" % name in text
    assert counts(text) == ((2 + 3) * 2, (1 + 0) * 2, 0, 2)      # stores: the block's 32-byte partial


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_stream_probe_hints_are_what_its_arguments_say(tmp_path):
    asm = assembly("ga_probe.hip", tmp_path)
    # stream_probe_kernel<R, W, KEEP, TILED>: the first KEEP inputs and outputs without the hint, all others with it
    for R, W, KEEP in ((5, 4, 0), (5, 4, 2), (2, 2, 2), (1, 1, 1), (4, 4, 1)):
        for tiled in (0, 1):
            text = kernel_text(asm, "19stream_probe_kernelILi%dELi%dELi%dELb%dEE" % (R, W, KEEP, tiled))
            assert counts(text) == (R - KEEP, KEEP, W - KEEP, KEEP), (R, W, KEEP, tiled)
