"""The boundary seen from plain C: include/novak.h must compile as C99 without warnings, the structs a C
compiler lays out must be the ones the ctypes binding mirrors, and the GPU-free entry points must
behave the same when called from C as through the binding."""
import ctypes as C
import os
import shutil
import subprocess

import pytest
import torch

from oracle import novak_oracle as O
from paper_2601_07876_amd import novak as N

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2601_07876_amd")


@pytest.fixture(scope="module")
def probe_output(tmp_path_factory):
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    N.load_library()                                   # fails loudly if the library is not built
    exe = str(tmp_path_factory.mktemp("c_abi") / "c_abi_probe")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi_probe.c"), "-o", exe, "-L", PKG, "-lnovak",
           "-Wl,--allow-shlib-undefined", "-Wl,-rpath," + PKG]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ)
    torch_lib = os.path.join(os.path.dirname(torch.__file__), "lib")      # the HIP runtime the library links to
    env["LD_LIBRARY_PATH"] = torch_lib + ":/opt/rocm/lib:" + env.get("LD_LIBRARY_PATH", "")
    out = subprocess.run([exe], check=True, capture_output=True, text=True, env=env, timeout=120).stdout
    return out.splitlines()


def _lines(out, prefix):
    return [l[len(prefix):].strip() for l in out if l.startswith(prefix)]


def test_struct_layout_matches_the_ctypes_mirror(probe_output):
    mirror = {"novak_hparams": N.novak_hparams, "novak_tensor_desc": N.novak_tensor_desc,
              "novak_step_scalars": N.novak_step_scalars, "novak_chunk": N.novak_chunk, "novak_info": N.novak_info}
    sizes = dict(l.split() for l in _lines(probe_output, "sizeof "))
    assert set(sizes) == set(mirror)
    for name, cls in mirror.items():
        assert int(sizes[name]) == C.sizeof(cls), name
    offsets = _lines(probe_output, "offset ")
    assert len(offsets) >= 25
    for l in offsets:
        path, off = l.split()
        struct, field = path.split(".")
        assert getattr(mirror[struct], field).offset == int(off), path


def test_host_entry_points_called_from_c(probe_output):
    out = probe_output
    # fast path: TRUE -> APPROX and BASIC -> MEMORY_EFFICIENT, with both warning bits (section 7.3)
    assert _lines(out, "validate rc ") == [f"0 nesterov {N.NOVAK_NESTEROV_APPROX} lookahead {N.NOVAK_LOOKAHEAD_MEMORY_EFFICIENT} warn 3"]
    assert _lines(out, "validate_bad rc ") == [str(N.NOVAK_ERR_INVALID_ARG)]
    # the prologue at t = 6 (first rectified step for beta2 = 0.999) against the oracle's scalars
    s = O.step_scalars(O.Hyper(), 6)
    vals = _lines(out, "scalars rc ")[0].split()
    assert vals[0] == "0" and int(vals[6]) == 1 and s.rectified_now
    assert float(vals[2]) == pytest.approx(s.rho_t, rel=1e-14) and float(vals[4]) == pytest.approx(s.r_t, rel=1e-13)
    assert float(vals[8]) == pytest.approx(1e-3 * s.r_t, rel=1e-13)
    # chunk planning of sizes (5, 0, 10000) with 4096-element chunks
    assert _lines(out, "plan rc ") == ["0 needed 4"]
    chunks = [tuple(int(x) for x in l.split()[2::2]) for l in _lines(out, "chunk ")]
    assert chunks == [(0, 0, 5), (2, 0, 4096), (2, 4096, 4096), (2, 8192, 1808)]
    assert _lines(out, "bytes ") == ["28.0 34.0"]
    # sizes (5, 0, 10000): tensors at 0, 256, 256; 10240 + 256 padded elements; 40.5 KiB -> 48 KiB + 2 KiB
    assert _lines(out, "arena rc ") == ["0 offsets 0 256 256 role_elems 10496 stride 51200"]
    assert _lines(out, "status ")[0] == N.novak_status_string(N.NOVAK_ERR_MISALIGNED)
    bad = _lines(out, "create_bad rc ")[0]
    assert bad.startswith(f"{N.NOVAK_ERR_INVALID_ARG} handle_null 1 msg ") and "device_id" in bad
    assert _lines(out, "destroy_null ") == ["0"]
