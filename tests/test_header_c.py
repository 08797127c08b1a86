"""include/sip.h is a C header: it must compile as plain C, and the structs that the Python
binding mirrors with ctypes must have the layout the binding assumes.  No GPU."""
import ctypes
import os
import subprocess
import sys
import tempfile

from paper_2506_22033_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INC = os.path.join(ROOT, "include")


def _run_c(source: str) -> str:
    with tempfile.TemporaryDirectory() as d:
        src, exe = os.path.join(d, "t.c"), os.path.join(d, "t")
        with open(src, "w") as f:
            f.write(source)
        subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", INC, "-o", exe, src],
                       check=True, capture_output=True, text=True)
        return subprocess.run([exe], check=True, capture_output=True, text=True).stdout


def test_header_compiles_as_c99_without_warnings():
    out = _run_c('#include "sip.h"\n#include <stdio.h>\nint main(void) { printf("%d %d\\n", (int)SIP_OK, (int)SIP_ERR_TIMEOUT); return 0; }\n')
    assert out.split() == ["0", str(binding.SIP_ERR_TIMEOUT)]


def test_diagnostic_header_compiles_as_c99_without_warnings():
    out = _run_c('#include "sip_diag.h"\n#include <stdio.h>\nint main(void) { printf("%d\\n", (int)SIP_OK); return 0; }\n')
    assert out.split() == ["0"]


def test_ctypes_mirrors_have_the_layout_of_the_c_structs():
    lines = ['#include "sip.h"', "#include <stdio.h>", "#include <stddef.h>", "int main(void) {",
             '  printf("params %zu\\n", sizeof(sip_params));', '  printf("call %zu\\n", sizeof(sip_call));']
    for name in binding.PARAM_FIELDS:
        lines.append(f'  printf("params.{name} %zu\\n", offsetof(sip_params, {name}));')
    for name, _ in binding.SipCall._fields_:
        lines.append(f'  printf("call.{name} %zu\\n", offsetof(sip_call, {name}));')
    lines += ["  return 0;", "}"]
    got = dict(l.split() for l in _run_c("\n".join(lines) + "\n").splitlines())
    assert int(got["params"]) == ctypes.sizeof(binding.SipParams)
    assert int(got["call"]) == ctypes.sizeof(binding.SipCall)
    for name in binding.PARAM_FIELDS:
        assert int(got[f"params.{name}"]) == getattr(binding.SipParams, name).offset, name
    for name, _ in binding.SipCall._fields_:
        assert int(got[f"call.{name}"]) == getattr(binding.SipCall, name).offset, name


def test_limits_in_the_binding_are_the_header_s():
    out = _run_c('#include "sip.h"\n#include <stdio.h>\nint main(void) { printf("%d %d %d %d %d\\n", SIP_MAX_V, '
                 'SIP_MAX_K_LOGPROBS, SIP_MAX_SHARDS, SIP_MAX_SLOTS, SIP_MAX_L); return 0; }\n')
    assert [int(x) for x in out.split()] == [binding.SIP_MAX_V, binding.SIP_MAX_K_LOGPROBS, binding.SIP_MAX_SHARDS,
                                              binding.SIP_MAX_SLOTS, binding.SIP_MAX_L]
