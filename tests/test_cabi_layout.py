"""CPU check: every ctypes mirror of an argument struct in the Python binding has the size and the field offsets
the C compiler gives the struct of include/lrnnx.h (a small C program compiled with gcc prints them)."""
import ctypes
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PAIRS = {
    "lrnnx_ss_fwd_args": "FwdArgs", "lrnnx_ss_fwd_complex_args": "FwdComplexArgs",
    "lrnnx_ss_bwd_args": "BwdArgs", "lrnnx_ss_bwd_complex_args": "BwdComplexArgs",
    "lrnnx_lti_args": "LtiArgs", "lrnnx_lti_bwd_args": "LtiBwdArgs",
    "lrnnx_diag_scan_args": "DiagScanArgs", "lrnnx_diag_scan_bwd_args": "DiagScanBwdArgs",
    "lrnnx_ss_step_args": "StepArgs", "lrnnx_ss_step_complex_args": "StepComplexArgs",
    "lrnnx_lti_step_args": "LtiStepArgs",
}


def test_ctypes_mirrors_match_the_header(tmp_path):
    pytest.importorskip("torch")
    from paper_2602_08810_amd import api
    lines = ['#include <stdio.h>', '#include <stddef.h>', f'#include "{ROOT}/include/lrnnx.h"', "int main(void) {"]
    for cname, pyname in PAIRS.items():
        lines.append(f'  printf("{cname} %zu\\n", sizeof({cname}));')
        for fname, _ in getattr(api, pyname)._fields_:
            lines.append(f'  printf("{cname}.{fname} %zu\\n", offsetof({cname}, {fname.rstrip("_")}));')
    lines += ["  return 0;", "}"]
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-o", str(exe), str(src)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    got = dict(line.split() for line in out.splitlines())
    for cname, pyname in PAIRS.items():
        cls = getattr(api, pyname)
        assert int(got[cname]) == ctypes.sizeof(cls), cname
        n_c_fields = sum(1 for k in got if k.startswith(cname + "."))
        assert n_c_fields == len(cls._fields_)
        for fname, _ in cls._fields_:
            assert int(got[f"{cname}.{fname}"]) == getattr(cls, fname).offset, f"{cname}.{fname}"


def test_header_has_no_field_the_binding_lacks():
    """The other direction: every field name in a struct of the header appears in its ctypes mirror."""
    import re
    pytest.importorskip("torch")
    from paper_2602_08810_amd import api
    text = open(os.path.join(ROOT, "include", "lrnnx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    for cname, pyname in PAIRS.items():
        body = re.search(r"typedef struct %s \{(.*?)\} %s;" % (cname, cname), text, flags=re.S).group(1)
        names = []
        for decl in body.split(";"):
            decl = decl.strip()
            if not decl:
                continue
            # "const void *u" / "int64_t u_stride_b, u_stride_d" / "int32_t B, D, N"
            first, *rest = decl.split(",")
            names.append(re.findall(r"[A-Za-z_][A-Za-z_0-9]*", first)[-1])
            names += [re.findall(r"[A-Za-z_][A-Za-z_0-9]*", r)[-1] for r in rest]
        have = [f.rstrip("_") for f, _ in getattr(api, pyname)._fields_]
        assert names == have, (cname, names, have)
