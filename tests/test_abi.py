"""The C-ABI library loads without a GPU, exports every function include/spec_tree.h declares, and
rejects on the host what the host can check (no kernel is launched by these calls)."""
import ctypes
import os
import re

import pytest

from paper_2305_09781_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "spec_tree.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spec_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTED)
    # the public header declares the method's calls (and their size queries, error text, version): no
    # measurement aids, and the library reads no environment variables
    assert not [n for n in names if "probe" in n or "debug" in n or "test" in n]
    csrc = os.path.join(ROOT, "paper_2305_09781_amd", "csrc")
    for f in os.listdir(csrc):
        assert "getenv" not in open(os.path.join(csrc, f)).read(), f
    for n in names:
        assert getattr(lib, n) is not None
    assert lib.spec_version() >= 100
    assert b"workspace" in lib.spec_strerror(binding.ERR_WORKSPACE)


def _desc(**kw):
    base = dict(B=1, H=4, H_kv=4, D=64, N=8, S_cap=136, dtype=binding.SPEC_F32, max_prefix_len=0,
                q_stride_b=8 * 4 * 64, q_stride_n=4 * 64, q_stride_h=64,
                kv_stride_b=4 * 136 * 64, kv_stride_h=136 * 64, kv_stride_s=64, new_stride_b=0, new_stride_n=0,
                new_stride_h=0, softmax_scale=0.0, plan_chunk_keys=0, plan_balanced_wgs=0, plan_heads_per_wg=0)
    base.update(kw)
    return binding.AttnDesc(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(), binding.ERR_INVALID_ARG),                       # null data pointers
    (dict(D=96), binding.ERR_UNSUPPORTED),
    (dict(N=129, S_cap=400), binding.ERR_UNSUPPORTED),
    (dict(H_kv=3), binding.ERR_UNSUPPORTED),                 # not a divisor of H
    (dict(H_kv=2, new_stride_b=8 * 2 * 64, new_stride_n=2 * 64, new_stride_h=32), binding.ERR_INVALID_ARG),
    (dict(dtype=5), binding.ERR_UNSUPPORTED),
    (dict(N=8, S_cap=4), binding.ERR_CAPACITY),
    (dict(max_prefix_len=130), binding.ERR_CAPACITY),
    (dict(q_stride_h=66), binding.ERR_INVALID_ARG),
    (dict(kv_stride_s=32), binding.ERR_INVALID_ARG),
    (dict(B=0), binding.ERR_INVALID_ARG),
    (dict(plan_chunk_keys=-1), binding.ERR_INVALID_ARG),
    (dict(plan_balanced_wgs=-2), binding.ERR_INVALID_ARG),
    (dict(plan_heads_per_wg=-1), binding.ERR_INVALID_ARG),
    (dict(S_cap=1 << 23, kv_stride_s=128, kv_stride_h=(1 << 23) * 128, kv_stride_b=4 * (1 << 23) * 128), binding.ERR_UNSUPPORTED),   # 4 GiB span
    (dict(softmax_scale=-1.0), binding.ERR_INVALID_ARG),
])
def test_attention_and_append_reject_bad_descriptors(kw, code):
    lib = binding.load()
    d = _desc(**kw)
    assert lib.spec_tree_attention(ctypes.byref(d), None, None, None, None, None, None, None, None, 0, None, None) == code
    assert lib.spec_kv_append(ctypes.byref(d), None, None, None, None, None, None, None) == code
    if kw:
        assert lib.spec_tree_attention_workspace_bytes(ctypes.byref(d)) == 0


def test_misaligned_pointers_and_workspace_are_rejected():
    lib = binding.load()
    d = _desc(S_cap=4104, kv_stride_h=4104 * 64, kv_stride_b=4 * 4104 * 64)   # long enough to be split
    buf = ctypes.create_string_buffer(4096)
    base = ctypes.addressof(buf)
    a = ctypes.c_void_p((base + 255) // 256 * 256)
    mis = ctypes.c_void_p(a.value + 4)
    assert lib.spec_tree_attention(ctypes.byref(d), mis, a, a, a, a, a, a, None, 0, None, None) == binding.ERR_INVALID_ARG
    need = lib.spec_tree_attention_workspace_bytes(ctypes.byref(d))
    assert need > 0
    assert lib.spec_tree_attention(ctypes.byref(d), a, a, a, a, a, a, a, None, 0, None, None) == binding.ERR_WORKSPACE
    assert lib.spec_tree_attention(ctypes.byref(d), a, a, a, a, a, a, a, a, need - 1, None, None) == binding.ERR_WORKSPACE


def test_static_scratch_entry_point_refuses_shapes_beyond_its_array():
    """The entry point that allocates nothing has a fixed scratch array: a launch plan that needs more is
    refused on the host (SPEC_ERR_WORKSPACE, nothing enqueued), a small one passes the size check."""
    lib = binding.load()
    B, H, D, N, S = 8, 8, 128, 128, 60128
    d = _desc(B=B, H=H, H_kv=H, D=D, N=N, S_cap=S, dtype=binding.SPEC_BF16, max_prefix_len=60000,
              q_stride_b=N * H * D, q_stride_n=H * D, q_stride_h=D, kv_stride_b=H * S * D, kv_stride_h=S * D, kv_stride_s=D)
    assert lib.spec_tree_attention_workspace_bytes(ctypes.byref(d)) > binding.STATIC_SCRATCH_BYTES
    buf = ctypes.create_string_buffer(4096)
    a = ctypes.c_void_p((ctypes.addressof(buf) + 255) // 256 * 256)
    assert lib.spec_tree_attention_append_static(ctypes.byref(d), a, a, a, a, a, a, a, a, a, None, None) == binding.ERR_WORKSPACE
    assert lib.spec_tree_attention_append_static(ctypes.byref(d), a, None, a, a, a, a, a, a, a, None, None) == binding.ERR_INVALID_ARG
    bad = _desc(D=96)
    assert lib.spec_tree_attention_append_static(ctypes.byref(bad), a, a, a, a, a, a, a, a, a, None, None) == binding.ERR_UNSUPPORTED


def test_verify_and_commit_reject_bad_arguments():
    lib = binding.load()
    assert lib.spec_verify_greedy(0, 8, 64, 0, None, None, None, 8, None, None, None, None, None, 0, None, None) == binding.ERR_INVALID_ARG
    assert lib.spec_verify_greedy(1, 200, 64, 0, None, None, None, 8, None, None, None, None, None, 0, None, None) == binding.ERR_UNSUPPORTED
    assert lib.spec_verify_greedy(1, 8, 64, 3, None, None, None, 8, None, None, None, None, None, 0, None, None) == binding.ERR_UNSUPPORTED
    assert lib.spec_verify_greedy(1, 8, 64, 0, None, None, None, 8, None, None, None, None, None, 0, None, None) == binding.ERR_INVALID_ARG
    assert lib.spec_verify_stochastic_workspace_bytes(2, 8, 64) >= 2 * 8 * 2 * 4 + 2 * 2 * 64 * 4
    assert lib.spec_verify_stochastic_workspace_bytes(0, 8, 64) == 0
    buf = ctypes.create_string_buffer(4096)
    a = ctypes.c_void_p((ctypes.addressof(buf) + 255) // 256 * 256)
    # temperature must be positive; workspace must be present
    assert lib.spec_verify_stochastic(1, 8, 64, 0, a, a, 1, a, a, a, a, a, a, 0.0, 8, a, a, a, a, 1 << 20, None, None) == binding.ERR_INVALID_ARG
    assert lib.spec_verify_stochastic(1, 8, 64, 0, a, a, 1, a, a, a, a, a, a, 1.0, 8, a, a, a, None, 0, None, None) == binding.ERR_WORKSPACE
    d = _desc()
    assert lib.spec_kv_commit(ctypes.byref(d), 0, None, None, None, 8, None, None, None, None, None) == binding.ERR_INVALID_ARG
    assert lib.spec_kv_commit(ctypes.byref(d), 200, None, None, None, 8, None, None, None, None, None) == binding.ERR_UNSUPPORTED
    arr = (ctypes.c_void_p * 1)(a.value)
    assert lib.spec_kv_commit(ctypes.byref(d), 1, arr, arr, a, 8, a, a, a, None, None) == binding.ERR_INVALID_ARG  # out aliases in


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libspectree.so")
    with pytest.raises(RuntimeError, match="not found"):
        binding.load()


def test_header_is_plain_c_and_links_from_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 with warnings as errors, and a C program that
    includes it links against the library and calls entry points that need no GPU."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "abi.c"
    src.write_text(
        '#include <stdio.h>\n#include <string.h>\n#include "spec_tree.h"\n'
        "int main(void) {\n"
        "  spec_attn_desc_t d; memset(&d, 0, sizeof d);\n"
        "  if (spec_version() < 100) return 1;\n"
        "  if (spec_kv_append(&d, 0, 0, 0, 0, 0, 0, 0) != SPEC_ERR_INVALID_ARG) return 2;\n"
        "  if (spec_tree_attention_workspace_bytes(&d) != 0) return 3;\n"
        '  if (strstr(spec_strerror(SPEC_ERR_WORKSPACE), "workspace") == 0) return 4;\n'
        '  printf("ok %d\\n", (int)sizeof(spec_attn_desc_t));\n  return 0;\n}\n')
    lib_dir = os.path.dirname(binding.lib_path())
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                    "-fsyntax-only", str(src)], check=True)
    exe = tmp_path / "abi"
    subprocess.run([gcc, "-std=c99", "-I", os.path.join(root, "include"), str(src), "-o", str(exe), "-L", lib_dir,
                    "-lspectree", "-Wl,-rpath," + lib_dir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    assert out.startswith("ok ") and int(out.split()[1]) == ctypes.sizeof(binding.AttnDesc)


def test_probe_library_exports_what_its_header_declares_and_checks_arguments():
    """libspecprobe (measurement aids, a library of its own): symbols of include/spec_probe.h, host-side checks."""
    from paper_2305_09781_amd import probe_binding
    text = open(os.path.join(ROOT, "include", "spec_probe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(spec_probe_[a-z_]+)\s*\(", text)))
    assert names == ["spec_probe_attention_traffic", "spec_probe_read_stream"]
    lib = probe_binding.load()
    for n in names:
        assert getattr(lib, n) is not None
    buf = ctypes.create_string_buffer(4096)
    a = ctypes.c_void_p((ctypes.addressof(buf) + 255) // 256 * 256)
    mis = ctypes.c_void_p(a.value + 4)
    f = lib.spec_probe_attention_traffic
    assert f(1, 1, 16, 16, 16, a, a, a, a, a, a, 15, None) == -1        # prefix + tree beyond the capacity
    assert f(1, 1, 129, 0, 256, a, a, a, a, a, a, 15, None) == -1       # more than 128 nodes
    assert f(1, 1, 16, 0, 32, a, mis, a, a, a, a, 15, None) == -1       # misaligned pointer
    assert f(1, 1, 16, 0, 32, a, a, None, a, a, a, 15, None) == -1      # null pointer
    assert f(1, 1, 16, 0, 32, a, a, a, a, a, a, 16, None) == -1         # unknown flag
    assert f(0, 1, 16, 0, 32, a, a, a, a, a, a, 15, None) == -1
    assert lib.spec_probe_read_stream(None, 64, a, None) == -1
