"""CPU-side checks of the boundary: the shared library loads without a GPU and exports every
symbol the header declares; host-side planning answers without touching a device."""
import os
import re

import pytest

from paper_2410_03090_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "uncomp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(uncomp_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    lib = binding.load_library()
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_workspace_query_runs_on_host():
    lib = binding.load_library()
    small = lib.uncomp_workspace_bytes(8, 1024, 128, 1, 8, 4, 32)
    big = lib.uncomp_workspace_bytes(256, 131072, 128, 32, 8, 4, 64)
    assert 0 < small < big
    assert lib.uncomp_workspace_bytes(0, 0, 128, 0, 0, 0, 0) > 0


def test_null_context_is_rejected_without_a_device():
    lib = binding.load_library()
    assert lib.uncomp_head_entropy(None, None, 0, 1, 1, 128, 0, 128, 32, 3, None, None, None) == binding.ERR_INVALID_ARG
    assert lib.uncomp_destroy(None) == binding.ERR_INVALID_ARG
    assert lib.uncomp_last_error(None) == b"null context"
    # the context-free entry point validates on the host before it touches a device, and leaves its reason
    assert lib.uncomp_head_entropy_noalloc(None, 0, 1, 1, 128, 0, 128, 32, 3, None, None, None) == binding.ERR_INVALID_ARG
    assert b"null pointer" in lib.uncomp_last_error(None)


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2410_03090_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+\S*oracle", src, flags=re.M), f
                assert "uncomp_oracle" not in src, f


def test_header_is_plain_c(tmp_path):
    """include/uncomp.h must be usable from C: a C99 translation unit that includes it and takes the
    address of every declared entry point compiles (syntax and types only; nothing is linked or run)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        import pytest
        pytest.skip("no C compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    from paper_2410_03090_amd import binding
    src = tmp_path / "use_header.c"
    body = "\n".join(f"    p[{i}] = (fn){name};" for i, name in enumerate(binding.EXPORTS))
    src.write_text('#include "uncomp.h"\ntypedef void (*fn)(void);\nvoid take(fn* p) {\n' + body + "\n}\n")
    r = subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I", os.path.join(root, "include"), str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
