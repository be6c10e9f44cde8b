"""The C-ABI library loads without a GPU and exports every function that
include/eep.h declares (no compute is called here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "eep.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(eep_[a-z_]+)\s*\(", text)))


def test_header_functions_are_exported():
    from paper_2605_10670_amd import binding
    names = declared_functions()
    assert {"eep_set_membership", "eep_update_placement", "eep_dispatch_layout", "eep_dispatch",
            "eep_combine"} <= set(names)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in eep.h but not exported"


def test_binding_resolves_and_reports_errors_without_gpu():
    from paper_2605_10670_amd import binding
    lib = binding.load()
    assert lib.eep_strerror(binding.ERR_COVERAGE).decode().startswith("a logical expert")
    assert lib.eep_destroy(None) == 0
    assert lib.eep_create(None, None) == binding.ERR_INVALID_ARG


def test_header_is_plain_c():
    import subprocess
    import tempfile
    with tempfile.TemporaryDirectory() as d:
        src = os.path.join(d, "t.c")
        open(src, "w").write('#include "eep.h"\nint main(void){eep_config c; (void)c; return 0;}\n')
        subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                        "-c", src, "-o", os.path.join(d, "t.o")], check=True)


def test_workspace_size_is_host_only_and_checks_the_config():
    from paper_2605_10670_amd import binding
    shape = dict(num_ranks=32, slots_per_rank=9, primary_slots=8, num_logical=256, max_tokens=4096,
                 topk=8, hidden=7168)
    n = binding.workspace_bytes(**shape)
    pairs = 4096 * 8
    assert n % 256 == 0 and n >= 3 * pairs * 4 + 2 * 32 * 288 * 4      # three pair arrays + tile counts
    assert n < 2 * (3 * pairs * 4 + 3 * 32 * 288 * 4 + 64 * 1024)      # and not much more
    assert binding.workspace_bytes(**dict(shape, max_tokens=8192)) > n
    with pytest.raises(binding.EepError) as ei:
        binding.workspace_bytes(**dict(shape, topk=0))
    assert ei.value.code == binding.ERR_INVALID_ARG
    with pytest.raises(binding.EepError) as ei:
        binding.workspace_bytes(**dict(shape, hidden=7))               # 14-byte rows
    assert ei.value.code == binding.ERR_ALIGN


def test_noalloc_scratch_size_is_host_only():
    from paper_2605_10670_amd import binding
    # decode shape: 32 tiles x 288 slots, two int matrices + two per-tile counters + header
    assert binding.noalloc_scratch_needed(32, 9, 4096) == 512 + 2 * 32 * 288 * 4 + 2 * 64 * 4
    assert binding.noalloc_scratch_needed(32, 9, 0) == 512
    assert binding.noalloc_scratch_needed(32, 9, 16384) < binding.NOALLOC_SCRATCH_BYTES
    assert binding.noalloc_scratch_needed(32, 9, 32 * 128 * 2048) > binding.NOALLOC_SCRATCH_BYTES
    with pytest.raises(binding.EepError):
        binding.noalloc_scratch_needed(32, 9, 33)
    # the header's constant and the binding's agree
    text = open(os.path.join(ROOT, "include", "eep.h")).read()
    assert "#define EEP_NOALLOC_SCRATCH_BYTES (4 * 1024 * 1024)" in text
