"""The C-ABI library loads and exports every symbol include/dash.h declares (no GPU needed),
and the binding refuses to work without the library or without a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dash_[a-z_0-9]+)\s*\(", text)))


def _lib():
    from paper_2302_06361_amd import binding
    if not os.path.exists(binding.lib_path()):
        from paper_2302_06361_amd import build
        build.build(force=True)
    return binding.lib(), binding


def test_header_declares_the_four_scheme_algorithms():
    names = _declared()
    for n in ("dash_garble_layer", "dash_eval_layer", "dash_encode", "dash_decode", "dash_input_labels",
              "dash_ctx_create", "dash_layer_sizes", "dash_weights_prepare"):
        assert n in names


def test_library_exports_every_declared_symbol():
    lib, binding = _lib()
    names = _declared()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.SYMBOLS) == names
    assert lib.dash_strerror(0) == b"ok" and lib.dash_strerror(-2) == b"size not supported"


def test_struct_layouts_match_the_header():
    """sizes the C compiler gives the two structs == what ctypes lays out"""
    import subprocess
    import tempfile
    from paper_2302_06361_amd import binding
    src = '#include <stdio.h>\n#include "dash.h"\nint main(){printf("%zu %zu %zu %zu\\n", sizeof(dash_labels), sizeof(dash_layer),' \
          ' offsetof(dash_layer, weights), offsetof(dash_layer, phi_stride));return 0;}\n'
    with tempfile.TemporaryDirectory() as d:
        open(os.path.join(d, "t.c"), "w").write(src)
        subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), "-o", os.path.join(d, "t"), os.path.join(d, "t.c")])
        out = subprocess.check_output([os.path.join(d, "t")]).split()
    assert int(out[0]) == ctypes.sizeof(binding.CLabels)
    assert int(out[1]) == ctypes.sizeof(binding.CLayer)
    assert int(out[2]) == binding.CLayer.weights.offset
    assert int(out[3]) == binding.CLayer.phi_stride.offset


def test_no_cpu_fallback():
    import torch
    from paper_2302_06361_amd import Context, DashError
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(DashError):
        Context([2, 3, 5], bytes(16))


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2302_06361_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)
