"""The C-ABI library builds for gfx950, loads without a GPU and exports every
symbol the public header declares; the ctypes mirror of the config struct has the
size the C compiler gives it.  No compute call is made here."""
import ctypes
import os
import re
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "sf_policy.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sf_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2006_11751_amd import binding
    if not os.path.exists(binding.library_path()):
        binding.build_library()
    lib = binding.load_library()
    names = _declared_functions()
    assert {"sf_policy_create", "sf_policy_step", "sf_policy_destroy", "sf_last_error"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(binding.EXPORTS) == set(names)
    assert binding.sf_last_error() == "" or isinstance(binding.sf_last_error(), str)


def test_struct_layout_matches_the_header():
    from paper_2006_11751_amd import binding
    src = ('#include <stdio.h>\n#include "sf_policy.h"\n'
           'int main(void){printf("%zu %zu %zu\\n", sizeof(sf_policy_config), sizeof(sf_policy_weights),'
           ' sizeof(sf_conv));return 0;}\n')
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "s.c")
        open(c, "w").write(src)
        exe = os.path.join(d, "s")
        subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), c, "-o", exe], check=True)
        sizes = [int(v) for v in subprocess.run([exe], capture_output=True, check=True).stdout.split()]
    assert sizes == [ctypes.sizeof(binding.SfPolicyConfig), ctypes.sizeof(binding.SfPolicyWeights),
                     ctypes.sizeof(binding.SfConv)]


def test_null_handle_calls_fail_cleanly_without_a_gpu():
    from paper_2006_11751_amd import binding
    lib = binding.load_library()
    assert lib.sf_policy_step(None, 1, None, None, None, None, 0, 0, None, None, None, None, None, None) == binding.SF_ERR_ARG
    assert "null handle" in binding.sf_last_error()
    assert lib.sf_policy_destroy(None) == binding.SF_OK
    assert lib.sf_policy_op_count(None) == 0
