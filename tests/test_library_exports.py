"""CPU-side checks of the boundary: the shared library loads without a GPU and exports every
symbol the header declares."""
import os
import re

import paper_1806_00588_amd as lsh
from paper_1806_00588_amd import binding, build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    if not os.path.exists(lsh.library_path()):
        hip_build.build(verbose=False)
    return lsh.load_library()


def test_header_symbols_are_all_exported():
    header = open(os.path.join(ROOT, "include", "lshbeam.h")).read()
    declared = set(re.findall(r"\b(lsh_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTED_SYMBOLS)
    lib = _lib()
    for sym in declared:
        assert getattr(lib, sym) is not None


def test_status_strings_and_kernel_names():
    lib = _lib()
    assert lib.lsh_status_string(0) == b"ok"
    assert lib.lsh_status_string(6) == b"workspace too small"
    assert lsh.kernel_names() == ["k_candidates", "k_logits", "k_select", "k_hit_rows", "k_part_bitmaps"]


def test_null_arguments_are_rejected_without_a_gpu():
    lib = _lib()
    assert lib.lsh_build_tables(None, None, None, None, None) == 1
    assert lib.lsh_decode_step(None, None, None, None, None, None, 0, None, None, None, None) == 1
    assert lib.lsh_step_workspace_bytes(None, None) == 0
    assert lib.lsh_decode_step_timed(None, None, None, None, None, None, 0, None, None, None, None,
                                     None) == 1
    assert lib.lsh_set_option(None, b"fused", 1) == 1
    assert lib.lsh_get_option(None, b"fused", None) == 1
    assert lib.lsh_profiler_create(0, None) == 1
    lib.lsh_profiler_destroy(None)
    lib.lsh_free_tables(None)


def test_decode_step_sources_never_read_the_environment():
    # launch-plan knobs are parsed once, when a handle is built; the step itself must not call
    # getenv (it is a hot call, and the environment is process-global state)
    src = open(os.path.join(ROOT, "paper_1806_00588_amd", "csrc", "lshbeam.hip")).read()
    assert src.count("std::getenv") == 1                      # inside env_int
    users = [m.start() for m in re.finditer(r"env_int\(", src)]
    step = src.index("lsh_status decode_step_impl(")
    step_end = src.index("}  // namespace", step)
    assert not any(step <= u < step_end for u in users)
    for name in os.listdir(os.path.join(ROOT, "paper_1806_00588_amd", "csrc")):
        if name.endswith(".h"):
            assert "getenv" not in open(os.path.join(ROOT, "paper_1806_00588_amd", "csrc", name)).read()


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1806_00588_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f
