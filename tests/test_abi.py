"""Host-side tests of the C ABI: the library loads without a GPU, exports every symbol the
header declares, and rejects invalid calls before any HIP call (so these run on a CPU machine)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ssd():
    from paper_2603_09555_amd import build
    build.build(force=False)
    from paper_2603_09555_amd import ssd as binding
    return binding


def declared_symbols(*headers):
    names = set()
    for h in headers:
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"SSD_API\s+[\w\s\*]+?\b(ssd_\w+)\s*\(", text))
    return sorted(names)


def exported_symbols(path):
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", path], check=True, capture_output=True, text=True).stdout
    return sorted(l.split()[-1] for l in out.splitlines() if " T " in l and l.split()[-1].startswith("ssd_"))


def test_header_symbols_are_exported(ssd):
    """The product library exports exactly what ssd.h and the test-only ssd_testing.h declare -- none of it
    creates events or waits -- and the measurement library adds exactly what ssd_measure.h declares."""
    names = declared_symbols("ssd.h", "ssd_testing.h")
    assert len(names) >= 7, names
    assert sorted(ssd.EXPORTS) == names
    assert exported_symbols(ssd.LIB_PATH) == names
    assert "ssd_prefill_profile" not in names and "ssd_peak_probe" not in names
    from paper_2603_09555_amd import measure
    extra = declared_symbols("ssd_measure.h")
    assert sorted(measure.EXPORTS) == extra == ["ssd_peak_probe", "ssd_prefill_profile"]
    assert exported_symbols(measure.LIB_PATH) == sorted(names + extra)


def test_header_is_plain_c_and_a_c_program_links(ssd, tmp_path):
    """The boundary is a C ABI: the header compiles as C99 with no C++ or HIP in sight, and a C program
    linked against the library can call the entry points that need no GPU (host-side validation)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    lib = os.path.join(root, "paper_2603_09555_amd", "libssd_hip.so")
    src = tmp_path / "use_ssd.c"
    src.write_text(r"""
#include <stdio.h>
#include "ssd.h"
int main(void) {
  ssd_shape s = {1, 2048, 24, 64, 128, 1, 256, SSD_BF16};
  size_t ws = ssd_prefill_workspace_bytes(&s);
  ssd_status st = ssd_prefill(&s, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL);
  s.nheads = 0;
  printf("%d %zu %d %zu %s|%s\n", ssd_version(), ws, (int)st, ssd_prefill_workspace_bytes(&s),
         ssd_prefill_path(&s), ssd_status_string(SSD_ERR_NULL));
  return 0;
}
""")
    exe = tmp_path / "use_ssd"
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(root, "include"), str(src), lib,
                    "-Wl,-rpath," + os.path.dirname(lib), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == ssd.version() and int(out[1]) > 0 and int(out[2]) == -1 and int(out[3]) == 0
    assert out[4].startswith("invalid|")


def test_version_and_status_strings(ssd):
    assert ssd.version() >= 100
    assert ssd.status_string(0) == "ok"
    for code in range(-7, 0):
        assert ssd.status_string(code) not in ("ok", "unknown status")
    assert ssd.status_string(-99) == "unknown status"


def shape(ssd, **kw):
    d = dict(batch=1, seqlen=64, nheads=4, headdim=32, dstate=16, ngroups=1, chunk=16, io_dtype=0)
    d.update(kw)
    return ssd.make_shape(**d)


def test_workspace_query(ssd):
    assert ssd.prefill_workspace_bytes(shape(ssd)) > 0
    assert ssd.prefill_workspace_bytes(shape(ssd)) % 256 == 0
    for bad in (dict(batch=0), dict(seqlen=0), dict(nheads=0), dict(headdim=-1), dict(dstate=0),
                dict(ngroups=0), dict(chunk=0), dict(nheads=6, ngroups=4), dict(io_dtype=2)):
        assert ssd.prefill_workspace_bytes(shape(ssd, **bad)) == 0, bad
        assert ssd.prefill_path(shape(ssd, **bad)) == "invalid"
    # seqlen need not be a multiple of chunk, and chunk may exceed seqlen
    assert ssd.prefill_workspace_bytes(shape(ssd, seqlen=65)) > 0
    assert ssd.prefill_workspace_bytes(shape(ssd, seqlen=5, chunk=64)) > 0
    assert ssd.prefill_path(shape(ssd)) in ("generic_f32", "mfma_f32", "mfma_bf16")


def test_prefill_rejects_before_any_hip_call(ssd):
    lib = ssd.raw()
    fake = ctypes.c_void_p(4096)  # never dereferenced: validation fails first
    ws = ctypes.c_void_p(4096)

    def call(s, x=fake, dt=fake, A=fake, B=fake, C=fake, D=fake, h0=None, y=fake, st=fake, w=ws, wb=1 << 40):
        return lib.ssd_prefill(ctypes.byref(s) if s is not None else None, x, dt, A, B, C, D, h0, y, st, w,
                               wb, None)

    assert call(None) == -1
    assert call(shape(ssd, batch=0)) == -2
    assert call(shape(ssd, nheads=6, ngroups=4)) == -2
    assert call(shape(ssd, io_dtype=7)) == -3
    assert call(shape(ssd), x=None) == -1
    assert call(shape(ssd), st=None) == -1
    assert call(shape(ssd), y=ctypes.c_void_p(4100)) == -7
    assert call(shape(ssd), h0=ctypes.c_void_p(4104)) == -7
    assert call(shape(ssd), w=None) == -5
    assert call(shape(ssd), wb=16) == -5
    assert call(shape(ssd), w=ctypes.c_void_p(4096 + 16)) == -5
    assert call(shape(ssd, batch=70000)) == -4
    assert call(shape(ssd, batch=2 ** 30, seqlen=2 ** 30)) == -2


def test_static_prefill_rejects_before_any_hip_call(ssd):
    """The entry point for callers that cannot allocate: invalid shapes, shapes whose scratch exceeds the
    library's static buffer and NULL tensors are refused on the host (no GPU needed to see it)."""
    import torch
    lib = ssd.raw()
    one = ctypes.c_void_p(256)
    ok = ssd.make_shape(1, 256, 4, 64, 128, 1, 64, torch.bfloat16)
    assert ssd.prefill_workspace_bytes(ok) <= ssd.STATIC_SCRATCH_BYTES
    args = [one] * 6 + [None, one, one, None]
    assert lib.ssd_prefill_static(None, *args) == -1
    bad = ssd.make_shape(1, 0, 4, 64, 128, 1, 64, torch.bfloat16)
    assert lib.ssd_prefill_static(ctypes.byref(bad), *args) == -2
    huge = ssd.make_shape(1, 16384, 80, 64, 128, 1, 256, torch.bfloat16)
    assert ssd.prefill_workspace_bytes(huge) > ssd.STATIC_SCRATCH_BYTES
    assert lib.ssd_prefill_static(ctypes.byref(huge), *args) == -8
    assert lib.ssd_prefill_static(ctypes.byref(ok), None, *args[1:]) == -1
    with open(os.path.join(ROOT, "include", "ssd.h")) as f:
        m = re.search(r"#define SSD_STATIC_SCRATCH_BYTES \(\(size_t\)(\d+) << (\d+)\)", f.read())
    assert m and int(m.group(1)) << int(m.group(2)) == ssd.STATIC_SCRATCH_BYTES


def test_knobs_do_not_change_workspace_sizes(ssd):
    """Forcing the generic kernel family changes which kernels run, never a size the caller was given."""
    import torch
    shapes = [ssd.make_shape(2, 1000, 8, 64, 128, 2, 128, torch.bfloat16), ssd.make_shape(1, 512, 4, 32, 16, 1, 64, torch.float32)]
    try:
        for sh in shapes:
            ssd.reset_knobs()
            a, av, path = ssd.prefill_workspace_bytes(sh), int(ssd.raw().ssd_prefill_varlen_workspace_bytes(ctypes.byref(sh))), ssd.prefill_path(sh)
            ssd.set_knob("force_generic", 1)
            assert ssd.prefill_path(sh) == "generic_f32"
            assert ssd.prefill_workspace_bytes(sh) == a
            assert int(ssd.raw().ssd_prefill_varlen_workspace_bytes(ctypes.byref(sh))) == av
            ssd.set_knob("seg_chunks", 1)
            assert ssd.prefill_workspace_bytes(sh) == a
            ssd.reset_knobs()
            assert ssd.prefill_path(sh) == path
        assert ssd.raw().ssd_testing_set_knob(99, 1) == -2
    finally:
        ssd.reset_knobs()


def test_decode_rejects_before_any_hip_call(ssd):
    lib = ssd.raw()
    fake = ctypes.c_void_p(4096)

    def call(s, nl=1, state=fake, x=fake, dt=fake, A=fake, B=fake, C=fake, D=fake, y=fake):
        return lib.ssd_decode_step_layers(nl, ctypes.byref(s) if s is not None else None, state, x, dt, A, B,
                                          C, D, y, None)

    assert call(None) == -1
    assert call(shape(ssd), nl=0) == -2
    assert call(shape(ssd, seqlen=0, chunk=0), state=None) == -1  # seqlen/chunk are ignored by decode
    assert call(shape(ssd, dstate=0)) == -2
    assert call(shape(ssd, io_dtype=-1)) == -3
    assert call(shape(ssd), state=ctypes.c_void_p(4100)) == -7
    assert call(shape(ssd), y=None) == -1
    assert lib.ssd_decode_step(ctypes.byref(shape(ssd)), None, fake, fake, fake, fake, fake, fake, fake,
                               None) == -1


def test_varlen_rejects_before_any_hip_call(ssd):
    lib = ssd.raw()
    fake = ctypes.c_void_p(4096)
    ok = dict(batch=3, seqlen=1000, nheads=8, headdim=64, dstate=128, ngroups=1, chunk=256, io_dtype=1)

    def call(s, cu=fake, x=fake, h0=None, w=fake, wb=1 << 40):
        return lib.ssd_prefill_varlen(ctypes.byref(s) if s is not None else None, cu, x, fake, fake, fake, fake, fake,
                                      h0, fake, fake, w, ctypes.c_size_t(wb), None)

    need = lib.ssd_prefill_varlen_workspace_bytes(ctypes.byref(shape(ssd, **ok)))
    assert need > 0 and need % 256 == 0
    assert call(None) == -1
    assert call(shape(ssd, **ok), cu=None) == -1
    assert call(shape(ssd, **ok), x=None) == -1
    assert call(shape(ssd, **ok), cu=ctypes.c_void_p(4098)) == -7
    assert call(shape(ssd, **ok), h0=ctypes.c_void_p(4100)) == -7
    assert call(shape(ssd, **ok), wb=need - 1) == -5
    assert call(shape(ssd, **ok), w=None) == -5
    assert call(shape(ssd, **dict(ok, seqlen=0))) == -2
    # outside the MFMA kernel family (fp32 io, other head shapes, chunk not a multiple of 64): the generic
    # kernels take the batch, so there is a workspace size for it
    for other in (dict(io_dtype=0), dict(headdim=32), dict(dstate=256), dict(dstate=100), dict(chunk=100),
                  dict(ngroups=4)):
        assert lib.ssd_prefill_varlen_workspace_bytes(ctypes.byref(shape(ssd, **dict(ok, **other)))) > 0
    # beyond what either family takes: sequences x heads over a grid axis, with fp32 io
    big = dict(ok, io_dtype=0, batch=9000, seqlen=20000)
    assert call(shape(ssd, **big)) == -4
    assert lib.ssd_prefill_varlen_workspace_bytes(ctypes.byref(shape(ssd, **big))) == 0


def test_prefill_dt_rejects_before_any_hip_call(ssd):
    lib = ssd.raw()
    fake = ctypes.c_void_p(4096)
    s = shape(ssd)
    need = lib.ssd_prefill_workspace_bytes(ctypes.byref(s))

    def call(xf, x=fake):
        return lib.ssd_prefill_dt(ctypes.byref(s), ctypes.byref(xf) if xf is not None else None, x, fake, fake, fake,
                                  fake, fake, None, fake, fake, fake, ctypes.c_size_t(need), None)

    assert call(None) == -1
    assert call(ssd.ssd_dt_transform(None, 1, 0.1, 0.01)) == -2     # dt_min > dt_max
    assert call(ssd.ssd_dt_transform(None, 1, 0.0, 0.0), x=None) == -1


def test_varlen_and_decode_dt_variants_reject_before_any_hip_call(ssd):
    lib = ssd.raw()
    fake = ctypes.c_void_p(4096)
    s = shape(ssd)
    need = lib.ssd_prefill_varlen_workspace_bytes(ctypes.byref(s))
    ok_xf = ssd.ssd_dt_transform(None, 1, 0.0, 0.0)
    bad_xf = ssd.ssd_dt_transform(None, 1, 0.1, 0.01)     # dt_min > dt_max

    def var(xf, x=fake):
        return lib.ssd_prefill_varlen_dt(ctypes.byref(s), ctypes.byref(xf) if xf is not None else None, fake, x, fake,
                                         fake, fake, fake, fake, None, fake, fake, fake, ctypes.c_size_t(need), None)

    def dec(xf, x=fake, nlayers=2):
        return lib.ssd_decode_step_layers_dt(nlayers, ctypes.byref(s), ctypes.byref(xf) if xf is not None else None,
                                             fake, x, fake, fake, fake, fake, fake, fake, None)

    def decs(xf, x=fake, nsteps=3):
        return lib.ssd_decode_steps_layers_dt(nsteps, 2, ctypes.byref(s), ctypes.byref(xf) if xf is not None else None,
                                              fake, x, fake, fake, fake, fake, fake, fake, None)

    for f in (var, dec, decs):
        assert f(None) == -1 and f(bad_xf) == -2 and f(ok_xf, x=None) == -1
        assert f(ok_xf, x=ctypes.c_void_p(4100)) == -7
    assert dec(ok_xf, nlayers=0) == -2 and decs(ok_xf, nsteps=0) == -2


def test_peak_probe_rejects_before_any_hip_call(ssd):
    from paper_2603_09555_amd import measure
    lib = measure.raw()
    fake = ctypes.c_void_p(4096)
    ms, work = ctypes.c_float(0), ctypes.c_double(0)

    def call(kind=1, iters=10, reps=1, a=fake, b=fake, nbytes=1 << 20, ms_=ctypes.byref(ms)):
        return lib.ssd_peak_probe(kind, iters, reps, a, b, ctypes.c_size_t(nbytes), ms_, ctypes.byref(work), None)

    assert call(ms_=None) == -1 and call(a=None) == -1 and call(b=None) == -1
    assert call(kind=7) == -2 and call(kind=-1) == -2 and call(reps=0) == -2 and call(nbytes=8) == -2
    assert call(kind=0, iters=0) == -2 and call(kind=0, nbytes=1024) == -2      # scratch too small for the MFMA loop
    assert call(a=ctypes.c_void_p(4100)) == -7


def test_conv_rejects_before_any_hip_call(ssd):
    lib = ssd.raw()
    fake = ctypes.c_void_p(4096)
    i3 = ctypes.c_int32 * 3

    def pre(batch=2, T=100, k=4, io=1, split=(64, 16, 16), u=fake, w=fake, z=(fake, fake, fake), sin=None, sout=fake,
            act=1):
        return lib.ssd_conv1d_prefill(batch, T, k, io, i3(*split) if split else None, u, w, None, sin, z[0], z[1], z[2],
                                      sout, act, None)

    assert pre(split=None) == -1
    assert pre(u=None) == -1 and pre(w=None) == -1
    assert pre(z=(fake, None, fake)) == -1
    assert pre(k=1) == -2 and pre(k=9) == -2 and pre(T=0) == -2 and pre(batch=0) == -2 and pre(act=2) == -2
    assert pre(split=(0, 8, 8)) == -2 and pre(split=(8, -1, 8)) == -2
    assert pre(io=5) == -3
    assert pre(u=ctypes.c_void_p(4100)) == -7 and pre(z=(fake, ctypes.c_void_p(4100), fake)) == -7
    assert pre(sin=fake, sout=fake) == -2   # the cache may not be updated in place by the prompt kernel
    st = lib.ssd_conv1d_step(2, 4, 1, i3(64, 16, 16), None, fake, fake, None, fake, fake, fake, 1, None)
    assert st == -1
    assert lib.ssd_conv1d_step(2, 4, 1, i3(64, 16, 16), fake, fake, fake, None, fake, None, fake, 1, None) == -1
    assert lib.ssd_conv1d_step(2, 4, 7, i3(64, 16, 16), fake, fake, fake, None, fake, fake, fake, 1, None) == -3


def test_decode_steps_rejects_before_any_hip_call(ssd):
    lib = ssd.raw()
    fake = ctypes.c_void_p(4096)

    def call(s, ns=2, nl=1, state=fake, x=fake, y=fake):
        return lib.ssd_decode_steps_layers(ns, nl, ctypes.byref(s) if s is not None else None, state, x, fake,
                                           fake, fake, fake, fake, y, None)

    assert call(None) == -1
    assert call(shape(ssd), ns=0) == -2
    assert call(shape(ssd), nl=0) == -2
    assert call(shape(ssd, headdim=0)) == -2
    assert call(shape(ssd), state=None) == -1
    assert call(shape(ssd), y=ctypes.c_void_p(4100)) == -7


def test_binding_fails_loudly_without_library(tmp_path, monkeypatch):
    """The product path has no fallback: with the .so absent the binding cannot be imported."""
    import importlib.util
    import shutil
    src = os.path.join(ROOT, "paper_2603_09555_amd", "ssd.py")
    dst = tmp_path / "ssd_copy.py"
    shutil.copy(src, dst)
    spec = importlib.util.spec_from_file_location("ssd_copy", str(dst))
    mod = importlib.util.module_from_spec(spec)
    with pytest.raises(ImportError):
        spec.loader.exec_module(mod)
