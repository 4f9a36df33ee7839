"""The C-ABI library loads without a GPU and exports every function include/he_mi355x.h declares;
the Python binding names the same set.  No compute call is made here."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "he_mi355x.h")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(he_[a-z0-9_]+)\s*\(", text)))


def test_header_functions_are_exported_and_bound():
    from paper_2302_02407_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2302_02407_amd.build import build_library
        build_library(verbose=False)
    lib = ctypes.CDLL(binding.LIB_PATH)
    names = _declared()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), "library does not export %s" % n
    assert sorted(binding.EXPORTS) == names


def test_header_compiles_as_plain_c(tmp_path):
    import subprocess
    src = tmp_path / "t.c"
    src.write_text('#include "he_mi355x.h"\nint main(void) { he_counters_t c; he_conv_plan p; he_raconv_plan r; (void)c; (void)p; (void)r; return HE_OK; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), "-c", str(src), "-o", str(tmp_path / "t.o")])


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2302_02407_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cuh")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f
    text = open(os.path.join(ROOT, "oracle", "he_oracle.py")).read() + open(os.path.join(ROOT, "oracle", "he_oracle.c")).read()
    assert "paper_2302_02407_amd" not in text
