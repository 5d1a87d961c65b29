"""The C-ABI library loads and exports every function the headers declare; host-only entry points
and argument checks behave as documented.  No kernel is launched here (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for hdr in os.listdir(os.path.join(ROOT, "include")):
        text = open(os.path.join(ROOT, "include", hdr)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(spec_\w+)\s*\(", text))
    return sorted(names)


@pytest.fixture(scope="module")
def lib():
    from paper_2411_00853_amd import binding
    return binding.lib()


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"spec_verify_init", "spec_verify_step", "spec_kv_rollback", "spec_verify_destroy",
            "spec_last_error"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/ but not exported"


def test_host_only_size_helpers(lib):
    from paper_2411_00853_amd import binding as sv
    from paper_2411_00853_amd import workload as wl
    assert sv.spec_packed_weight_bytes(4096, 4096) == 4096 * 4096 * 2
    assert sv.spec_packed_weight_bytes(100, 64) == 7 * 4 * 1024        # 7 row tiles x (2 -> 4) K blocks x 1 KiB
    assert sv.spec_packed_weight_bytes(64, 100) == 0                   # n_in must be a multiple of 32
    cfg = sv.make_cfg(wl.SEVEN_B, 8, 2048 + 6, 5)
    # 32 layers x 8 slots x 32 heads x 2080 (padded) positions x 128 dims x (k,v) x 2 bytes
    assert sv.spec_kv_cache_bytes(cfg) == 32 * 8 * 32 * 2080 * 128 * 2 * 2
    tiny = sv.make_cfg(wl.TINY, 1, 133, 4)
    assert sv.spec_kv_cache_bytes(tiny) == 2 * 1 * 4 * 133 * 64 * 2 * 4


def test_bad_configurations_are_rejected_before_any_device_work(lib):
    from paper_2411_00853_amd import binding as sv
    from paper_2411_00853_amd import workload as wl
    out = C.c_void_p()
    assert lib.spec_verify_init(None, None, None, 0, None, C.byref(out)) == -1
    assert b"cfg" in lib.spec_last_error()
    bad = sv.make_cfg(wl.SEVEN_B, 300, 2054, 5)                       # max_batch above the limit
    assert lib.spec_verify_init(C.byref(bad), None, None, 0, None, C.byref(out)) == -1
    bad = sv.make_cfg(wl.SEVEN_B, 8, 2054, 16)                        # lookahead above the limit
    assert lib.spec_verify_init(C.byref(bad), None, None, 0, None, C.byref(out)) == -1
    odd = sv.make_cfg(wl.ModelShape(1, 64, 3, 2, 64, 64, 100), 1, 64, 2)   # 3 q heads over 2 kv heads
    assert sv.spec_kv_cache_bytes(odd) == 0
    assert lib.spec_verify_step(None, None, None, None) == -1
    assert lib.spec_kv_rollback(None, None, None, 0, None) == -1


def test_noalloc_step_refuses_sizes_beyond_its_fixed_workspace(lib):
    """Host-side checks of spec_sample_step_noalloc come before any device work."""
    from paper_2411_00853_amd import binding as sv
    ks = (C.c_int32 * 65)()
    dummy = C.c_void_p(16)      # never dereferenced: the size checks come first
    out = sv.spec_step_out(dummy, dummy, None)
    for vocab, kmax, batch in ((1000, 4, 65), (262145, 4, 2), (1000, 16, 2), (0, 4, 2)):
        args = sv.spec_step_args(batch, ks, None, None, dummy, dummy, dummy, 1.0, dummy, 0)
        assert lib.spec_sample_step_noalloc(vocab, kmax, C.byref(args), C.byref(out), None) == -2
        assert b"outside" in lib.spec_last_error()
    args = sv.spec_step_args(2, ks, None, None, dummy, dummy, dummy, 1.0, None, 0)     # no target_logits_in
    assert lib.spec_sample_step_noalloc(1000, 4, C.byref(args), C.byref(out), None) == -1


def test_build_lists_name_existing_sources():
    """Every source the build compiles exists, and per-source options refer to listed sources."""
    import os
    from paper_2411_00853_amd import build as b
    for src in b.SOURCES:
        assert os.path.exists(os.path.join(b.CSRC, src)), src
    assert set(b.SOURCE_FLAGS) <= set(b.SOURCES)
    assert "--offload-arch=gfx950" in b.FLAGS and "-packed-fp32-ops" in b.FLAGS


def test_headers_are_plain_c_and_the_binding_mirrors_their_structs(tmp_path):
    """The three headers compile as strict C11 (no C++ needed to call the library), and every struct the
    Python binding marshals has the size and field offsets the C compiler gives it."""
    import ctypes as C
    import subprocess
    from paper_2411_00853_amd import binding as sv
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    names = ["spec_model_cfg", "spec_layer_weights", "spec_weights", "spec_step_args", "spec_step_out",
             "spec_tree_args", "spec_tree_out", "spec_decode_cfg", "spec_round_args", "spec_lookahead_cfg",
             "spec_decode_view", "spec_step_plan"]
    lines = ['#include <stddef.h>', '#include <stdio.h>', '#include "spec_verify.h"', '#include "spec_decode.h"',
             '#include "spec_kernels.h"', 'int main(void) {']
    for n in names:
        cls = getattr(sv, n)
        lines.append(f'  printf("{n} size %zu\\n", sizeof({n}));')
        for f, _ in cls._fields_:
            lines.append(f'  printf("{n} {f} %zu\\n", offsetof({n}, {f}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines) + "\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(root, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    seen = 0
    for line in out:
        if not line:
            continue
        n, f, v = line.split()
        cls = getattr(sv, n)
        want = C.sizeof(cls) if f == "size" else getattr(cls, f).offset
        assert int(v) == want, line
        seen += 1
    assert seen == sum(len(getattr(sv, n)._fields_) + 1 for n in names)
    # and the limits the binding or the tests rely on are the header's
    text = open(os.path.join(root, "include", "spec_verify.h")).read()
    for macro, value in (("SPEC_MAX_BATCH", 256), ("SPEC_MAX_LOOKAHEAD", 15), ("SPEC_MAX_STEP_ROWS", 352),
                         ("SPEC_NOALLOC_MAX_BATCH", 64), ("SPEC_NOALLOC_MAX_VOCAB", 262144)):
        assert f"#define {macro} {value}" in text, macro
