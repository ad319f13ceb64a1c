"""The C-ABI library loads, exports every symbol include/co2.h declares, and
rejects bad arguments on the host before anything is enqueued (no GPU needed:
every call here fails validation, so no kernel is launched and no pointer is
dereferenced)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2401_16265_amd as co2

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "co2.h")
LAYOUT_HEADER = os.path.join(os.path.dirname(HEADER), "co2_layout.h")


def declared_functions():
    src = open(HEADER).read() + open(LAYOUT_HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(co2_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"co2_outer_step", "co2_pseudo_grad_norms", "co2_inner_adamw", "co2_workspace_bytes",
            "co2_strerror"} <= set(names)
    L = co2.lib()
    assert os.path.samefile(co2.lib_path(), os.path.join(os.path.dirname(co2.__file__), "libco2.so"))
    for n in names:
        assert hasattr(L, n), f"libco2.so does not export {n}"


def test_params_struct_layout_matches_header():
    # field order in the header == field order in the ctypes mirror
    src = open(HEADER).read()
    body = re.search(r"typedef struct co2_params \{(.*?)\} co2_params;", src, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"([A-Za-z_][A-Za-z0-9_]*)\s*;", body)
    assert fields == [f[0] for f in co2.Co2Params._fields_]
    assert C.sizeof(co2.Co2Params) == 8 + 4 + 4 + 8 + 8 + 16 + 4 + 4 + 8 + 8 + 8 + 8 + 4 + 4


def test_strerror_and_workspace_bytes():
    for code in (0, -1, -2, -3, -99):
        assert isinstance(co2.strerror(code), str) and co2.strerror(code)
    assert co2.workspace_bytes(0, 1, 1) == 0
    assert co2.workspace_bytes(10, 0, 1) == 0
    assert co2.workspace_bytes(10, 1, 17) == 0
    w1 = co2.workspace_bytes(1 << 20, 8, 4)
    w2 = co2.workspace_bytes(1 << 24, 8, 4)
    assert 0 < w1 < w2 and w1 % 256 == 0
    # bounded: a quarter of a byte per element (two regions of 32-byte records per 256 elements)
    assert co2.workspace_bytes(1343868928, 292, 8) < 1343868928 // 4 + (1 << 20)


A = 0x7F0000000000          # fake, 256-byte aligned "device" addresses: never dereferenced
NB = 4096 * 4


def _fake(i):
    return A + i * (1 << 20)


def _params(seg, **kw):
    seg = np.asarray(seg, dtype=np.int64)
    d = dict(n=int(seg[-1]), S=len(seg) - 1, K=2, seg_off=seg.ctypes.data, seg_off_dev=_fake(20),
             alpha=1.0, beta=0.9, clip_phi=1.0, penalty_c=1.0, tau=4, flags=0, step=1)
    d.update(kw)
    return co2.Co2Params(**d), seg


def _call(p, params=_fake(0), anchor=_fake(1), anchor_out=_fake(1), momentum=_fake(2),
          deltas=(_fake(3), _fake(4)), delta_out=_fake(5), fsn=None, lam=None, ws=_fake(8),
          ws_bytes=1 << 19):
    dp = (C.c_void_p * len(deltas))(*deltas) if deltas is not None else None
    return co2.lib().co2_outer_step(C.byref(p), params, anchor, anchor_out, momentum, dp,
                                    delta_out, fsn, lam, ws, ws_bytes, None)


@pytest.mark.parametrize("bad", [
    dict(K=0), dict(K=17), dict(tau=0), dict(step=-1), dict(beta=1.0), dict(beta=-0.1),
    dict(clip_phi=0.0), dict(clip_phi=-1.0), dict(clip_phi=float("nan")), dict(penalty_c=-1.0),
    dict(alpha=float("inf")), dict(alpha=float("nan")), dict(flags=16), dict(seg_off_dev=None),
    dict(sweep_waves_per_cu=-1), dict(sweep_waves_per_cu=33),
    dict(flags=4, pull_rho=0.0), dict(flags=4, pull_rho=1.5), dict(flags=4, pull_rho=float("nan")),
    dict(flags=2, penalty_c=1.0),                 # current-round order with a penalty needs first-step norms
    dict(S=0), dict(n=0), dict(n=4095), dict(flags=1, step=0),
])
def test_outer_step_rejects_bad_hyperparameters(bad):
    p, keep = _params([0, 1000, 4096], **bad)
    assert _call(p) == co2.CO2_EINVAL


def test_outer_step_rejects_bad_tables():
    for seg in ([1, 10, 4096], [0, 3000, 2000, 4096]):
        p, keep = _params(seg)
        assert _call(p) == co2.CO2_EINVAL


def test_outer_step_rejects_bad_buffers():
    p, keep = _params([0, 1000, 4096])
    assert _call(p, anchor=None) == co2.CO2_EINVAL
    assert _call(p, momentum=None) == co2.CO2_EINVAL
    assert _call(p, params=None) == co2.CO2_EINVAL                    # delta_out without params
    assert _call(p, delta_out=None) == co2.CO2_EINVAL
    assert _call(p, deltas=None) == co2.CO2_EINVAL
    assert _call(p, deltas=(_fake(3), None)) == co2.CO2_EINVAL
    assert _call(p, params=_fake(0) + 4) == co2.CO2_EINVAL            # misaligned
    assert _call(p, deltas=(_fake(3) + 8, _fake(4))) == co2.CO2_EINVAL
    assert _call(p, momentum=_fake(0) + 1024) == co2.CO2_EINVAL       # overlaps params
    assert _call(p, delta_out=_fake(4)) == co2.CO2_EINVAL             # output on a peer's delta
    assert _call(p, delta_out=_fake(3) + 16) == co2.CO2_EINVAL        # partly on deltas[0] (all of it is allowed)
    assert _call(p, anchor_out=_fake(1) + 16) == co2.CO2_EINVAL       # partial overlap with anchor
    assert _call(p, deltas=(_fake(2), _fake(4))) == co2.CO2_EINVAL    # delta is the momentum
    assert _call(p, ws=None) == co2.CO2_EWORKSPACE
    assert _call(p, ws=_fake(8) + 16) == co2.CO2_EWORKSPACE
    assert _call(p, ws_bytes=128) == co2.CO2_EWORKSPACE
    assert _call(p, ws=_fake(2)) == co2.CO2_EINVAL                    # workspace on the momentum
    # carried norms need a previous delta_out when no first_step_norm is given
    p2, keep2 = _params([0, 1000, 4096], flags=1)
    assert _call(p2, params=None, delta_out=None, anchor_out=_fake(6)) == co2.CO2_EINVAL


def test_static_entry_point_validates_like_the_workspace_one():
    """co2_outer_step_static checks its arguments before it touches the GPU."""
    def call(p, params=_fake(0), anchor=_fake(1), momentum=_fake(2), deltas=(_fake(3), _fake(4)),
             delta_out=_fake(5)):
        dp = (C.c_void_p * len(deltas))(*deltas)
        return co2.lib().co2_outer_step_static(C.byref(p), params, anchor, anchor, momentum, dp,
                                               delta_out, None, None, None)
    p, keep = _params([0, 1000, 4096], K=0)
    assert call(p) == co2.CO2_EINVAL
    p, keep = _params([0, 1000, 4096])
    assert call(p, momentum=_fake(0) + 1024) == co2.CO2_EINVAL
    assert call(p, delta_out=_fake(4)) == co2.CO2_EINVAL
    # sizes whose partial sums do not fit the static scratch array
    big = 200_000_000
    assert co2.workspace_bytes(big, 2, 2) > co2.CO2_STATIC_SCRATCH_BYTES
    p, keep = _params([0, 1000, big])
    assert call(p) == co2.CO2_ESCRATCH
    assert "scratch" in co2.strerror(co2.CO2_ESCRATCH)
    src = open(HEADER).read()
    assert re.search(r"#define\s+CO2_STATIC_SCRATCH_BYTES\s+\(32u << 20\)", src)
    assert co2.CO2_STATIC_SCRATCH_BYTES == 32 << 20


def test_norms_and_adamw_reject_bad_arguments():
    L = co2.lib()
    p, keep = _params([0, 1000, 4096])
    bufs = (C.c_void_p * 2)(_fake(3), _fake(4))
    assert L.co2_pseudo_grad_norms(C.byref(p), bufs, 2, None, None, _fake(8), 1 << 19, None) == co2.CO2_EINVAL
    assert L.co2_pseudo_grad_norms(C.byref(p), bufs, 33, None, _fake(9), _fake(8), 1 << 19, None) == co2.CO2_EINVAL
    assert L.co2_pseudo_grad_norms(C.byref(p), None, 0, None, _fake(9), _fake(8), 1 << 19, None) == co2.CO2_EINVAL
    assert L.co2_pseudo_grad_norms(C.byref(p), bufs, 2, None, _fake(9), _fake(8), 64, None) == co2.CO2_EWORKSPACE
    assert L.co2_pseudo_grad_norms(None, bufs, 2, None, _fake(9), _fake(8), 1 << 19, None) == co2.CO2_EINVAL

    def adam(n=4096, p_in=_fake(0), p_out=_fake(0), g=_fake(1), m=_fake(2), v=_fake(3), lr=3e-4,
             b1=0.9, b2=0.95, eps=1e-8, wd=0.1, k=1, anchor=None, dout=None, seg=None, segd=None,
             S=0, sq=None, ws=None, wsb=0):
        return L.co2_inner_adamw(n, p_in, p_out, g, m, v, lr, b1, b2, eps, wd, k, anchor, dout,
                                 seg, segd, S, sq, ws, wsb, None)

    assert adam(n=0) == co2.CO2_EINVAL
    assert adam(k=0) == co2.CO2_EINVAL
    assert adam(g=None) == co2.CO2_EINVAL
    assert adam(b1=1.0) == co2.CO2_EINVAL
    assert adam(anchor=_fake(4)) == co2.CO2_EINVAL                    # anchor without delta_out
    assert adam(m=_fake(0)) == co2.CO2_EINVAL                         # exp_avg on the params
    assert adam(p_out=_fake(0) + 64) == co2.CO2_EINVAL                # partial overlap p_in/p_out
    assert adam(sq=_fake(5)) == co2.CO2_EINVAL                        # norm without a table
    assert adam(p_out=None) == co2.CO2_EINVAL                         # p' stored nowhere (no delta_out either)
    assert adam(sq=_fake(5), seg=keep.ctypes.data, segd=_fake(20), S=2, ws=_fake(8), wsb=16) == co2.CO2_EWORKSPACE
    assert L.co2_sqrt_to_f32(None, _fake(1), 4, None) == co2.CO2_EINVAL
    assert L.co2_copy_f32(_fake(0), _fake(0), 16, None) == co2.CO2_EINVAL


def test_binding_fails_loudly_without_the_library(tmp_path, monkeypatch):
    """No CPU fallback: if libco2.so is absent and cannot be built, loading raises."""
    import subprocess

    from paper_2401_16265_amd import binding, build
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(build, "LIB_PATH", str(tmp_path / "libco2.so"))
    monkeypatch.setenv("HIPCC", "/bin/false")
    with pytest.raises((subprocess.CalledProcessError, OSError)):
        binding.lib()
    monkeypatch.undo()
    assert binding.lib() is not None


def test_package_does_not_import_the_oracle():
    import subprocess
    import sys
    code = ("import sys; import paper_2401_16265_amd, paper_2401_16265_amd.schedule; "
            "bad=[m for m in sys.modules if m.startswith('oracle')]; sys.exit(1 if bad else 0)")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    assert subprocess.run([sys.executable, "-c", code], cwd=root).returncode == 0


def test_outer_step_bf16_validates_like_the_fp32_entry():
    p, keep = _params([0, 1000, 4096])
    L = co2.lib()
    dp = (C.c_void_p * 2)(_fake(3), _fake(4))
    ok_args = [C.byref(p), _fake(0), _fake(1), _fake(1), _fake(2), dp, _fake(5), None, None, _fake(8), 1 << 19, None]
    bad = list(ok_args); bad[6] = None                       # delta_out missing
    assert L.co2_outer_step_bf16(*bad) == co2.CO2_EINVAL
    bad = list(ok_args); bad[6] = _fake(3) + 4096            # overlaps deltas[0] (2-byte elements: 8 KiB)
    assert L.co2_outer_step_bf16(*bad) == co2.CO2_EINVAL
    bad = list(ok_args); bad[9] = None
    assert L.co2_outer_step_bf16(*bad) == co2.CO2_EWORKSPACE


def test_header_is_plain_c(tmp_path):
    """include/co2.h must be usable from C (no C++-only constructs, no HIP/torch types)."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "co2.h"\n#include "co2_layout.h"\n'
                   "int main(void) { co2_params p; co2_buffer_set* b = 0; p.n = 1; (void)p; (void)b; "
                   "return (int)co2_workspace_bytes(0, 0, 0) + (co2_strerror(0) == 0); }\n")
    inc = os.path.dirname(HEADER)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", inc, "-c", str(src),
                    "-o", str(tmp_path / "use_header.o")], check=True)
    text = open(HEADER).read() + open(LAYOUT_HEADER).read()
    # the compute header declares nothing that allocates, and the library has no hidden
    # configuration channel: no source file reads the environment
    plain = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    assert "create" not in plain and "destroy" not in plain
    csrc = os.path.join(os.path.dirname(co2.__file__), "csrc")
    for f in os.listdir(csrc):
        assert "getenv" not in open(os.path.join(csrc, f)).read(), f
    for forbidden in ("torch", "hipStream_t ", "#include <hip", "at::Tensor"):
        assert forbidden not in text.replace("a hipStream_t;", "")


def test_buffer_set_rejects_bad_arguments():
    """Validation precedes every HIP call, so these return without touching a device."""
    L = co2.lib()
    one = (C.c_size_t * 1)(4096)
    zero = (C.c_size_t * 1)(0)
    out = (C.c_void_p * 1)()
    handle = C.c_void_p()
    mib = 1 << 20
    assert L.co2_buffer_set_create(0, one, 0, out, C.byref(handle)) == co2.CO2_EINVAL
    assert L.co2_buffer_set_create(co2.CO2_MAX_BUFFER_SET + 1, one, 0, out, C.byref(handle)) == co2.CO2_EINVAL
    assert L.co2_buffer_set_create(1, None, 0, out, C.byref(handle)) == co2.CO2_EINVAL
    assert L.co2_buffer_set_create(1, one, 0, None, C.byref(handle)) == co2.CO2_EINVAL
    assert L.co2_buffer_set_create(1, one, 0, out, None) == co2.CO2_EINVAL
    assert L.co2_buffer_set_create(1, zero, 0, out, C.byref(handle)) == co2.CO2_EINVAL
    assert L.co2_buffer_set_create(1, one, mib, out, C.byref(handle)) == co2.CO2_EINVAL     # not a 2 MiB multiple
    assert L.co2_buffer_set_create(1, one, 3 * mib, out, C.byref(handle)) == co2.CO2_EINVAL
    assert L.co2_buffer_set_destroy(None) == co2.CO2_EINVAL
    assert not handle.value
    src = open(LAYOUT_HEADER).read()
    assert int(re.search(r"#define CO2_MAX_BUFFER_SET (\d+)", src).group(1)) == co2.CO2_MAX_BUFFER_SET
