"""The C-ABI library loads without a GPU, exports every symbol the header declares, and its
argument structs have the layout the Python binding marshals into."""
import ctypes as C
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "cascade_verify.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2605_07230_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2605_07230_amd import build
        build.build(verbose=False)
    return binding.load_library()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"^\s*(?:const\s+char\s*\*|int64_t|int)\s+(\w+)\s*\(", text, flags=re.M)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2605_07230_amd import binding
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layout_matches_the_header(tmp_path):
    from paper_2605_07230_amd import binding
    src = tmp_path / "sizes.c"
    structs = ["cascade_limits", "tree_attn_args", "lmhead_args", "accept_args", "select_args", "kv_commit_args", "conv_weight_args"]
    body = "\n".join(f'  printf("{s} %zu\\n", sizeof({s}));' for s in structs)
    probes = [("tree_attn_args", "lse"), ("tree_attn_args", "cache_stride_row"), ("lmhead_args", "row_lse"),
              ("accept_args", "n_conv"), ("select_args", "tvd_used"), ("select_args", "eps_tvd"),
              ("kv_commit_args", "cache_stride_layer"), ("kv_commit_args", "prefix_len_out"),
              ("conv_weight_args", "cos_next"), ("accept_args", "feature_space"), ("select_args", "draft_dist")]
    body += "\n" + "\n".join(f'  printf("{s}.{f} %zu\\n", offsetof({s}, {f}));' for s, f in probes)
    src.write_text(f'#include <stdio.h>\n#include <stddef.h>\n#include "{HEADER}"\nint main(void) {{\n{body}\n  return 0;\n}}\n')
    exe = tmp_path / "sizes"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", str(src), "-o", str(exe)])
    out = dict(line.split() for line in subprocess.check_output([str(exe)], text=True).splitlines())
    for s in structs:
        assert int(out[s]) == C.sizeof(getattr(binding, s)), s
    for s, f in probes:
        assert int(out[f"{s}.{f}"]) == getattr(getattr(binding, s), f).offset, (s, f)


def test_host_side_errors_without_a_gpu(lib):
    from paper_2605_07230_amd import binding
    assert lib.cascade_strerror(0) == b"ok"
    assert b"dtype" in lib.cascade_strerror(binding.EDTYPE)
    # null arguments are rejected before anything touches the device
    assert lib.tree_verify_attn(None, None) == binding.EINVAL
    assert lib.lmhead_softmax_cfg(None, None) == binding.EINVAL
    assert lib.cascade_accept(None, None) == binding.EINVAL
    assert lib.select_path(None, None) == binding.EINVAL
    assert lib.kv_commit(None, None) == binding.EINVAL
    assert lib.convergence_weights(None, None) == binding.EINVAL
    assert lib.cascade_measure_mfma_bf16(None, 1, None) == binding.EINVAL
    assert lib.cascade_measure_hbm_read(None, None, 0, 1, None) == binding.EINVAL
    assert lib.cascade_destroy(None) == binding.EINVAL
    assert lib.cascade_device_status(None) == binding.EINVAL
    handle = C.c_void_p(1234)
    assert lib.cascade_create(C.byref(handle), None, None) == binding.EINVAL and not handle.value
    bad = binding.cascade_limits(1, 10, 2000, 16, 8, 64, 512, 4096)       # tree larger than the library maximum
    assert lib.cascade_create(C.byref(handle), C.byref(bad), None) == binding.ESHAPE and not handle.value
    bad = binding.cascade_limits(1, 10, 10, 16, 8, 64, 512, 1 << 20)      # vocabulary too large
    assert lib.cascade_create(C.byref(handle), C.byref(bad), None) == binding.ESHAPE
    bad = binding.cascade_limits(0, 10, 10, 16, 8, 64, 512, 4096)
    assert lib.cascade_create(C.byref(handle), C.byref(bad), None) == binding.EINVAL


def test_missing_library_raises(monkeypatch, tmp_path):
    from paper_2605_07230_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError):
        binding.load_library()
