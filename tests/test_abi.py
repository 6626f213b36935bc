"""Host-side checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching a device.  No
compute call is made here (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def api():
    lib = os.path.join(ROOT, "paper_2602_12675_amd", "libsla2.so")
    if not os.path.exists(lib):
        from paper_2602_12675_amd.build import build_library
        build_library(verbose=False)
    from paper_2602_12675_amd import api
    return api


def header_functions():
    src = open(os.path.join(ROOT, "include", "sla2.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(sla2_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(api):
    names = header_functions()
    assert set(names) == set(api.EXPORTS)
    lib = ctypes.CDLL(api.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert api.sla2_version() >= 1


def test_struct_sizes_match_header(api):
    assert ctypes.sizeof(api.Params) == 12 * 4 + 6 * 8
    assert ctypes.sizeof(api.WsLayout) == 20 * ctypes.sizeof(ctypes.c_size_t)


def test_num_selected_and_workspace(api):
    p = api.make_params(1, 12, 32760, 128, 128, 64, 0.03)
    assert api.sla2_num_selected(p) == 15
    p.topk_frac = 0.05
    assert api.sla2_num_selected(p) == 26
    p = api.make_params(1, 40, 75600, 128, 128, 64, 0.03)
    assert api.sla2_num_selected(p) == 35
    p = api.make_params(1, 2, 1024, 64, 64, 64, 0.125, dtype=api.SLA2_F32)
    assert api.sla2_num_selected(p) == 2
    L = api.sla2_workspace_layout(p)
    assert L.total == api.sla2_workspace_bytes(p) > 0
    offs = [getattr(L, n) for n, _ in api.WsLayout._fields_]
    assert all(o % 256 == 0 for o in offs)
    assert offs == sorted(offs)


@pytest.mark.parametrize("kw,status", [
    (dict(d=96), "EUNSUPPORTED"), (dict(block_q=32), "EUNSUPPORTED"), (dict(block_kv=128), "EUNSUPPORTED"),
    (dict(topk_frac=1.5), "EINVAL"), (dict(topk_frac=-0.1), "EINVAL"), (dict(topk_frac=float("nan")), "EINVAL"),
    (dict(N=0), "EINVAL"), (dict(B=0), "EINVAL"), (dict(dtype=7), "EINVAL"), (dict(quant_mode=4), "EINVAL"), (dict(quant_mode=-1), "EINVAL"),
    (dict(flags=8), "EINVAL"), (dict(N=64 * 2048 + 1), "EUNSUPPORTED"),
    (dict(dtype=0, quant_mode=1), "EUNSUPPORTED"), (dict(dtype=0, quant_mode=2), "EUNSUPPORTED"),
    (dict(dtype=0, quant_mode=3), "EUNSUPPORTED"),
])
def test_bad_parameters_are_rejected_on_the_host(api, kw, status):
    base = dict(B=1, H=2, N=1024, d=64, block_q=64, block_kv=64, topk_frac=0.125, dtype=api.SLA2_BF16)
    base.update(kw)
    p = api.make_params(**base)
    assert api.sla2_workspace_bytes(p) == 0
    # pointers are never dereferenced on the host: dummy non-null addresses are enough
    rc = api.sla2_forward(p, 256, 256, 256, 256, 256, 4096, workspace=None, check=False)
    assert rc == getattr(api, "SLA2_" + status)
    assert api.sla2_strerror(rc) != "unknown status"


def test_null_alias_and_workspace_errors(api):
    p = api.make_params(1, 2, 1024, 64, 64, 64, 0.125, dtype=api.SLA2_F32)
    need = api.sla2_workspace_bytes(p)
    lib = ctypes.CDLL(api.LIB_PATH)
    lib.sla2_forward.restype = ctypes.c_int
    vp = ctypes.c_void_p
    lib.sla2_forward.argtypes = [ctypes.POINTER(api.Params)] + [vp] * 9 + [ctypes.c_size_t, vp]
    tensor = 1 * 2 * 1024 * 64 * 4
    q, k, v, out = 1 << 20, 2 << 20, 3 << 20, 4 << 20
    ws = 16 << 20
    ok_args = [q, k, v, 256, 512, out, None, None, ws, need, None]

    def call(args):
        return lib.sla2_forward(ctypes.byref(p), *args)
    a = list(ok_args); a[0] = None
    assert call(a) == api.SLA2_EINVAL
    a = list(ok_args); a[5] = None
    assert call(a) == api.SLA2_EINVAL
    a = list(ok_args); a[5] = q + tensor - 16          # out overlaps the end of q
    assert call(a) == api.SLA2_EALIAS
    a = list(ok_args); a[5] = v
    assert call(a) == api.SLA2_EALIAS
    a = list(ok_args); a[8] = None
    assert call(a) == api.SLA2_EWORKSPACE
    a = list(ok_args); a[9] = need - 1
    assert call(a) == api.SLA2_EWORKSPACE
    a = list(ok_args); a[8] = ws + 8                   # misaligned
    assert call(a) == api.SLA2_EWORKSPACE


@pytest.mark.parametrize("kw,status", [
    (dict(in_stride=(0, 64, 64)), "EINVAL"),                       # partly set
    (dict(in_stride=(-1, 64 * 1024, 64)), "EINVAL"),
    (dict(in_stride=(2 * 1024 * 64, 1024 * 64, 32)), "EUNSUPPORTED"),    # token stride below d
    (dict(in_stride=(2 * 1024 * 68, 1024 * 68, 68)), "EUNSUPPORTED"),    # 136-byte rows: not a multiple of 16 bytes
    (dict(out_stride=(2 * 1024 * 64, 60, 2 * 64)), "EUNSUPPORTED"),      # head stride not a multiple of 16 bytes
    (dict(in_stride=(1 << 40, 64, 1 << 24)), "EUNSUPPORTED"),            # token stride too large
])
def test_bad_strides_are_rejected_on_the_host(api, kw, status):
    p = api.make_params(1, 2, 1024, 64, 64, 64, 0.125, dtype=api.SLA2_BF16, **kw)
    assert api.sla2_workspace_bytes(p) == 0
    rc = api.sla2_forward(p, 256, 256, 256, 256, 256, 1 << 30, workspace=None, check=False)
    assert rc == getattr(api, "SLA2_" + status)


def test_strided_alias_and_alignment_checks(api):
    # [B, N, H, d] views of a packed projection: spans of q, k, v interleave, out may not touch them
    B, H, N, d = 1, 2, 1024, 64
    st = (N * 3 * H * d, d, 3 * H * d)
    p = api.make_params(B, H, N, d, 64, 64, 0.125, dtype=api.SLA2_BF16, in_stride=st, out_stride=(N * H * d, d, H * d))
    need = api.sla2_workspace_bytes(p)
    assert need > 0
    base, ws = 1 << 20, 64 << 20
    q, k, v = base, base + H * d * 2, base + 2 * H * d * 2
    span = ((N - 1) * st[2] + (H - 1) * st[1] + d) * 2
    assert api.sla2_forward(p, q, k, v, 256, 256, q + span - 16, workspace=ws, ws_bytes=need, check=False) == api.SLA2_EALIAS
    assert api.sla2_forward(p, q, k, v, 256, 256, q + 8, workspace=ws, ws_bytes=need, check=False) == api.SLA2_EINVAL
    assert api.sla2_forward(p, q + 2, k, v, 256, 256, 1 << 30, workspace=ws, ws_bytes=need, check=False) == api.SLA2_EINVAL


def test_backward_gradient_slices_may_interleave_but_not_share_elements(api):
    # dq, dk, dv as slices of one packed [B, N, 3, H, d] gradient buffer are fine as far as the host checks go
    # (that call would go on to launch, so only the refusals are exercised here): shifted by half a row they
    # share elements with their neighbour and must be refused, as must a gradient on top of an input
    B, H, N, d = 1, 2, 1024, 64
    st = (N * 3 * H * d, d, 3 * H * d)
    p = api.make_params(B, H, N, d, 64, 64, 0.125, dtype=api.SLA2_BF16, in_stride=st, out_stride=(N * H * d, d, H * d),
                        flags=api.SLA2_FLAG_SAVE_FOR_BACKWARD)
    need = api.sla2_workspace_bytes(p)
    assert need > 0
    base, gbase, ws = 1 << 20, 1 << 26, 1 << 28
    q, k, v = base, base + H * d * 2, base + 2 * H * d * 2
    dq, dk, dv = gbase, gbase + H * d * 2, gbase + 2 * H * d * 2
    go = 1 << 27

    def call(dq_, dk_, dv_):
        return api.sla2_backward(p, q, k, v, 256, go, dq_, dk_, dv_, 512, ws, ws_bytes=need, check=False)

    assert call(dq, dq + 32, dv) == api.SLA2_EALIAS            # dk starts inside head 0's dq rows
    assert call(dq, dk, dk + (H - 1) * d * 2) == api.SLA2_EALIAS
    assert call(q, dk, dv) == api.SLA2_EALIAS                  # a gradient on top of an input
    assert call(dq, dk, go) == api.SLA2_EALIAS


# ---- the header, compiled as plain C, against the ctypes mirror -------------------------------- #
_C_PROBE = r"""
#include <stdio.h>
#include <stddef.h>
#include "sla2.h"
#define FIELD(S, f) printf("field " #S " " #f " %zu %zu\n", offsetof(S, f), sizeof(((S*)0)->f))
#define ENUM(e) printf("enum " #e " %d\n", (int)(e))
int main(void) {
  printf("sizeof sla2_params %zu\n", sizeof(sla2_params));
  printf("sizeof sla2_ws_layout %zu\n", sizeof(sla2_ws_layout));
@BODY@
  return 0;
}
"""


def _header_struct_fields(name):
    src = open(os.path.join(ROOT, "include", "sla2.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    body = re.search(r"typedef struct %s \{(.*?)\} %s;" % (name, name), src, flags=re.S).group(1)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        names = re.sub(r"^(unsigned|long long|size_t|int|float)\s+", "", decl)
        fields += [re.sub(r"\[.*\]", "", n).strip() for n in names.split(",")]
    return fields


def _header_enumerators():
    src = open(os.path.join(ROOT, "include", "sla2.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = []
    for body in re.findall(r"typedef enum \{(.*?)\}", src, flags=re.S):
        names += re.findall(r"\b(SLA2_[A-Z0-9_]+)\b", body)
    names += re.findall(r"#define (SLA2_(?:FLAG|STATIC)_[A-Z0-9_]+)", src)
    return names


def test_header_compiles_as_c_and_matches_the_binding(api, tmp_path):
    """include/sla2.h must be a plain C header (no HIP, no C++), and every field offset, field size,
    struct size and enumerator value the C compiler sees must be what the ctypes binding assumes."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    pf, wf, en = _header_struct_fields("sla2_params"), _header_struct_fields("sla2_ws_layout"), _header_enumerators()
    lines = ["  FIELD(sla2_params, %s);" % f for f in pf] + ["  FIELD(sla2_ws_layout, %s);" % f for f in wf] + \
            ["  ENUM(%s);" % e for e in en]
    src = tmp_path / "probe.c"
    src.write_text(_C_PROBE.replace("@BODY@", "\n".join(lines)))
    exe = tmp_path / "probe"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    seen_fields, seen_enums, sizes = {}, {}, {}
    for ln in out:
        t = ln.split()
        if not t:
            continue
        if t[0] == "field":
            seen_fields[(t[1], t[2])] = (int(t[3]), int(t[4]))
        elif t[0] == "enum":
            seen_enums[t[1]] = int(t[2])
        else:
            sizes[t[1]] = int(t[2])
    # structs: same field names in the same order, same offsets and sizes
    for cname, cls, names in (("sla2_params", api.Params, pf), ("sla2_ws_layout", api.WsLayout, wf)):
        assert [n for n, _ in cls._fields_] == names
        assert ctypes.sizeof(cls) == sizes[cname]
        for n in names:
            fld = getattr(cls, n)
            assert (fld.offset, fld.size) == seen_fields[(cname, n)], (cname, n)
    # enumerators and flags: the binding's constants of the same name, and the stage order
    for name, val in seen_enums.items():
        if name.startswith("SLA2_STAGE_"):
            continue
        assert getattr(api, name) == val, name
    stages = {n[len("SLA2_STAGE_"):].lower(): v for n, v in seen_enums.items() if n.startswith("SLA2_STAGE_")}
    assert stages.pop("count") == len(api.STAGES)
    assert {n: i for i, n in enumerate(api.STAGES)} == stages
    assert api.QUANT_MODES == {"none": seen_enums["SLA2_QUANT_NONE"], "fp8": seen_enums["SLA2_QUANT_FP8"],
                               "int8": seen_enums["SLA2_QUANT_INT8"], "fp8v": seen_enums["SLA2_QUANT_FP8_V"]}
