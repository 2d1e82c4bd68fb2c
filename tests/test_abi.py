"""The shared library builds for gfx950, loads without a GPU and exports every entry point
the public header declares (no compute calls here)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "aero.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(aero_[a-z_]+)\s*\(", text)))


def library():
    from paper_2602_14338_amd import binding, build
    if not os.path.exists(binding.library_path()):
        build.build()
    return binding.library_path()


def test_header_declares_the_four_calls():
    names = declared_functions()
    for n in ("aero_group_advantage", "aero_logprob_fwd", "aero_grpo_loss_bwd", "aero_lmhead_logprob_fused",
              "aero_workspace_bytes", "aero_status_string"):
        assert n in names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(library())
    for n in declared_functions():
        assert hasattr(lib, n), n


def test_status_strings_and_workspace_sizes_on_host():
    import paper_2602_14338_amd as aero
    from paper_2602_14338_amd import binding
    lib = ctypes.CDLL(library())
    lib.aero_status_string.restype = ctypes.c_char_p
    seen = {lib.aero_status_string(i) for i in range(8)}
    assert len(seen) == 8 and lib.aero_status_string(99) == b"unknown status"
    assert aero.aero_workspace_bytes(binding.OP_GROUP_ADVANTAGE, T=10) == 0
    assert aero.aero_workspace_bytes(binding.OP_LOGPROB_FWD, T=10, V=100) == 0
    a = aero.aero_workspace_bytes(binding.OP_GRPO_LOSS_BWD, T=16384, V=151936)
    assert a % 256 == 0 and 16384 * 4 * 5 <= a <= 16384 * 4 * 10
    f4 = aero.aero_workspace_bytes(binding.OP_LMHEAD_FUSED, T=16384, V=151936, H=1536)
    f5 = aero.aero_workspace_bytes(binding.OP_LMHEAD_FUSED, T=32768, V=152064, H=3584)
    assert 0 < f4 < 16 << 30 and f4 < f5 < 32 << 30      # both layouts of the bf16 dz are held whole


def test_binding_has_no_cpu_fallback():
    src = open(os.path.join(ROOT, "paper_2602_14338_amd", "binding.py")).read()
    assert "oracle" not in src and "numpy" not in src


def test_header_is_plain_c_and_its_constants_match_the_binding(tmp_path):
    """include/aero.h compiles as C99 on its own, and every constant the binding re-states has the
    header's value."""
    import subprocess
    from paper_2602_14338_amd import binding
    names = ["AERO_F32", "AERO_BF16", "AERO_F16", "AERO_F8E4M3", "AERO_ROW_PADDING", "AERO_ROW_UNTOUCHED",
             "AERO_OP_GROUP_ADVANTAGE", "AERO_OP_LOGPROB_FWD", "AERO_OP_GRPO_LOSS_BWD", "AERO_OP_LMHEAD_FUSED",
             "AERO_NOALLOC_MAX_T", "AERO_DW_ACCUMULATE"]
    src = tmp_path / "consts.c"
    src.write_text('#include "aero.h"\n#include <stdio.h>\nint main(void) {\n' +
                   "".join('  printf("%s %%ld\\n", (long)%s);\n' % (n, n) for n in names) +
                   '  printf("sizeof_params %ld\\n", (long)sizeof(aero_adv_params));\n  return 0;\n}\n')
    exe = tmp_path / "consts"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    got = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True,
                                                       text=True).stdout.splitlines())
    assert int(got["AERO_F32"]) == binding.AERO_F32 and int(got["AERO_BF16"]) == binding.AERO_BF16
    assert int(got["AERO_F16"]) == binding.AERO_F16
    assert int(got["AERO_ROW_PADDING"]) == binding.AERO_ROW_PADDING == -1
    assert int(got["AERO_ROW_UNTOUCHED"]) == binding.AERO_ROW_UNTOUCHED == -2
    assert int(got["AERO_F8E4M3"]) == binding.AERO_F8E4M3
    assert [int(got[n]) for n in names[6:10]] == [binding.OP_GROUP_ADVANTAGE, binding.OP_LOGPROB_FWD,
                                                 binding.OP_GRPO_LOSS_BWD, binding.OP_LMHEAD_FUSED]
    assert int(got["sizeof_params"]) == ctypes.sizeof(binding._AdvParamsC)
    assert int(got["AERO_NOALLOC_MAX_T"]) == 65536
    assert int(got["AERO_DW_ACCUMULATE"]) == binding.AERO_DW_ACCUMULATE == 0x100
