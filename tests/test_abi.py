"""CPU-side checks of the C ABI: the library loads, exports every function the header declares, the ctypes
mirrors of the structs have the C layout, and argument errors are reported without touching a GPU."""
import ctypes as C
import os
import re
import subprocess
import tempfile

import pytest

import focus_inputs as fi
import paper_2601_23278_amd as pk
from paper_2601_23278_amd import binding
from paper_2601_23278_amd.runner import config_from_workload

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "focus.h")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(focus_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert {"focus_init", "focus_prefill_kv", "focus_step", "focus_free"} <= set(names)
    lib = C.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names                 # the binding covers the same set


def test_struct_layouts_match_the_header():
    prog = r'''
#include <stdio.h>
#include <stddef.h>
#include "focus.h"
int main(void) {
  printf("%zu %zu %zu %zu\n", sizeof(focus_config), sizeof(focus_weights), sizeof(focus_step_out), sizeof(focus_seq_state));
  printf("%zu %zu %zu %zu\n", offsetof(focus_config, rms_eps), offsetof(focus_config, keep_ratio),
         offsetof(focus_config, conf_threshold), offsetof(focus_seq_state, tokens));
  printf("%zu %zu\n", offsetof(focus_step_out, logits), offsetof(focus_weights, w_down));
  return 0;
}'''
    with tempfile.TemporaryDirectory() as d:
        open(os.path.join(d, "t.c"), "w").write(prog)
        subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                               os.path.join(d, "t.c"), "-o", os.path.join(d, "t")])
        out = subprocess.check_output([os.path.join(d, "t")]).decode().split()
    got = [int(x) for x in out]
    exp = [C.sizeof(pk.focus_config), C.sizeof(binding.focus_weights), C.sizeof(pk.focus_step_out), C.sizeof(pk.focus_seq_state),
           pk.focus_config.rms_eps.offset, pk.focus_config.keep_ratio.offset, pk.focus_config.conf_threshold.offset,
           pk.focus_seq_state.tokens.offset, pk.focus_step_out.logits.offset, binding.focus_weights.w_down.offset]
    assert got == exp


def good_cfg():
    return config_from_workload(fi.workload("c1_tiny"), 4, 64, 24)


def test_sizes_and_config_errors_without_gpu():
    c = good_cfg()
    assert pk.focus_workspace_bytes(c) > 0
    assert pk.focus_kv_pool_bytes(c) == 2 * 24 * 2 * 4 * 16 * 64 * 4
    for field, bad in [("head_dim", 96), ("block_size", 65), ("block_size", 0), ("n_kv_heads", 3), ("dtype", 7),
                       ("evict_layer", 0), ("evict_layer", 2), ("maxpool_k", 5), ("budget_mode", 4), ("constraints", 4),
                       ("mask_token_id", 1024), ("hidden", 100), ("n_pages", 0)]:
        c = good_cfg()
        setattr(c, field, bad)
        with pytest.raises(pk.FocusError) as e:
            pk.focus_workspace_bytes(c)
        assert e.value.code == binding.FOCUS_EINVAL, field


def test_selection_and_expert_config_errors_without_gpu():
    moe = dict(n_experts=8, experts_per_token=2, expert_ffn=64, shared_ffn=32, first_moe_layer=1, route_scale=1.0)

    def cfg(**over):
        c = good_cfg()
        for k, v in {**moe, **over}.items():
            setattr(c, k, v)
        return c
    dense = pk.focus_workspace_bytes(good_cfg())
    assert pk.focus_workspace_bytes(cfg()) > dense                       # the expert work buffers are planned
    assert pk.focus_workspace_bytes(cfg(n_experts=0, experts_per_token=99)) == dense   # dense model: the rest is ignored
    for over in [dict(n_experts=513), dict(n_experts=-1), dict(experts_per_token=0), dict(experts_per_token=9),
                 dict(n_experts=64, experts_per_token=33), dict(expert_ffn=60), dict(shared_ffn=-8), dict(first_moe_layer=3),
                 dict(route_scale=0.0), dict(selection=3), dict(selection=-1), dict(intra_block_cache=2)]:
        with pytest.raises(pk.FocusError) as e:
            pk.focus_workspace_bytes(cfg(**over))
        assert e.value.code == binding.FOCUS_EINVAL, over
    lib = binding._lib
    assert lib.focus_run_steps(None, None, 1, None, 1, 1, None, None) == binding.FOCUS_EINVAL
    assert lib.focus_set_route_override(None, None) == binding.FOCUS_EINVAL


def test_init_rejects_null_and_reports_text():
    lib = binding._lib
    ctx = C.c_void_p()
    c = good_cfg()
    rc = lib.focus_init(C.byref(c), None, None, 0, None, 0, C.byref(ctx))
    assert rc == binding.FOCUS_EINVAL and b"null" in lib.focus_last_error(None)
    assert lib.focus_step(None, None, 1, None, None, None, None) == binding.FOCUS_EINVAL
    assert lib.focus_free(None) == binding.FOCUS_OK


def test_binding_fails_loudly_without_the_library_and_never_touches_the_oracle(tmp_path):
    """The product path has no fallback: with libfocus.so out of reach the import raises, and neither the binding nor
    the runner imports anything from oracle/."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2601_23278_amd")
    # a copy of the package's Python files without the built library
    dst = tmp_path / "paper_2601_23278_amd"
    dst.mkdir()
    for f in os.listdir(pkg):
        if f.endswith(".py"):
            (dst / f).write_text(open(os.path.join(pkg, f)).read())
    code = "import sys; sys.path.insert(0, %r); sys.path.insert(1, %r)\ntry:\n    import paper_2601_23278_amd\nexcept ImportError as e:\n    print('IMPORT-ERROR', e)\n" % (str(tmp_path), root)
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120).stdout
    assert "IMPORT-ERROR" in out and "libfocus.so is not built" in out
    for f in ("binding.py", "runner.py", "__init__.py", "build.py"):
        src = open(os.path.join(pkg, f)).read()
        assert "oracle" not in src, f
    csrc = os.path.join(pkg, "csrc")
    for f in os.listdir(csrc):
        text = open(os.path.join(csrc, f)).read()
        assert "oracle/" not in text and not [l for l in text.splitlines() if l.startswith("#include") and "oracle" in l], f
