"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol
the header declares, and rejects bad arguments before anything touches a device.
No compute call is made here (there is no GPU in this environment)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2102_08374_amd as P
from paper_2102_08374_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
lib = binding._lib

OK, EINVAL, EALIGN, ERANGE, EHIP, EWORKSPACE, ENOPLAN = 0, -1, -2, -3, -4, -5, -6
FAKE = 0x7F0000001000        # aligned, never dereferenced: validation fails first
FAKE_ODD = FAKE + 4


def declared_functions():
    text = open(os.path.join(ROOT, "include", "intsgd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(intsgd_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 16
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTED_SYMBOLS) == names


def test_python_binding_has_the_same_names():
    for name in declared_functions():
        if name == "intsgd_last_hip_error":
            continue
        assert hasattr(P, name), name


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2102_08374_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                where = os.path.join(dirpath, f)
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), where
                assert not re.search(r"liboracle|oracle/|oracle_[a-z]+\s*\(", text), where


def ptrs(n, value=FAKE):
    return (C.c_void_p * n)(*[value + 0x1000 * i for i in range(n)])


def call_step_fused(desc, grads=None, alpha=FAKE, eta=0.1, x=FAKE, ns=FAKE, sat=FAKE, ws=FAKE,
                    ws_bytes=1 << 40):
    n = max(1, min(desc.c.n, 128))
    g = ptrs(n) if grads is None else grads
    return lib.intsgd_step_fused(desc.ref(), g, alpha, eta, x, ns, sat, ws, ws_bytes, None)


def test_descriptor_validation():
    good = dict(d=1000, n=4)
    assert P.intsgd_workspace_bytes(P.Desc(**good)) > 0
    bad = [
        (dict(d=0, n=4), EINVAL), (dict(d=1000, n=0), EINVAL), (dict(d=1000, n=129), ERANGE),
        (dict(d=1 << 41, n=1), ERANGE),
        (dict(d=1000, n=4, clip=0), ERANGE), (dict(d=1000, n=4, clip=-3), ERANGE),
        (dict(d=1000, n=4, clip=(2**31 - 1) // 4 + 1), ERANGE),
        (dict(d=1000, n=4, wire=8, clip=128), ERANGE),
        (dict(d=1000, n=4, rounding=2), EINVAL), (dict(d=1000, n=4, wire=16), EINVAL),
        (dict(d=1000, n=4, block_offsets=[0, 10, 10, 1000]), EINVAL),
        (dict(d=1000, n=4, block_offsets=[0, 500, 400, 1000]), EINVAL),
        (dict(d=1000, n=4, block_offsets=[1, 500, 1000]), EINVAL),
        (dict(d=1000, n=4, block_offsets=[0, 500, 999]), EINVAL),
    ]
    for kw, want in bad:
        desc = P.Desc(**kw)
        assert P.intsgd_workspace_bytes(desc) == 0, kw
        assert call_step_fused(desc) == want, kw
        assert lib.intsgd_prepare(desc.ref()) == want, kw
    # B > 1 without offsets, and B > d
    desc = P.Desc(**good)
    desc.c.num_blocks = 3
    assert call_step_fused(desc) == EINVAL
    assert lib.intsgd_step_fused(None, ptrs(1), FAKE, 0.1, FAKE, FAKE, FAKE, FAKE, 1 << 40, None) == EINVAL


def test_pointer_alignment_eta_and_workspace_validation():
    desc = P.Desc(1000, 4)
    need = P.intsgd_workspace_bytes(desc)
    assert call_step_fused(desc, grads=None, x=None) == EINVAL
    assert call_step_fused(desc, x=FAKE_ODD) == EALIGN
    assert call_step_fused(desc, grads=ptrs(4, FAKE_ODD)) == EALIGN
    g = ptrs(4)
    g[2] = None
    assert call_step_fused(desc, grads=g) == EINVAL
    assert lib.intsgd_step_fused(desc.ref(), None, FAKE, 0.1, FAKE, FAKE, FAKE, FAKE, need, None) == EINVAL
    assert call_step_fused(desc, alpha=None) == EINVAL
    assert call_step_fused(desc, ns=None) == EINVAL
    assert call_step_fused(desc, sat=None) == EINVAL
    for eta in (0.0, -0.1, float("nan"), float("inf")):
        assert call_step_fused(desc, eta=eta) == EINVAL
    assert call_step_fused(desc, ws=None) == EWORKSPACE
    assert call_step_fused(desc, ws=FAKE + 16) == EWORKSPACE
    assert call_step_fused(desc, ws_bytes=need - 1) == EWORKSPACE
    # the other entry points share the same checks
    assert lib.intsgd_compress(desc.ref(), ptrs(4), FAKE, ptrs(4, FAKE_ODD), FAKE, FAKE, need, None) == EALIGN
    assert lib.intsgd_compress(desc.ref(), ptrs(4), FAKE, ptrs(4), None, FAKE, need, None) == EINVAL
    assert lib.intsgd_int_sum(desc.ref(), ptrs(4), FAKE_ODD, None) == EALIGN
    assert lib.intsgd_int_sum(desc.ref(), None, FAKE, None) == EINVAL
    assert lib.intsgd_decode_update(desc.ref(), FAKE, FAKE, -1.0, FAKE, None, None) == EINVAL
    assert lib.intsgd_decode_update(desc.ref(), FAKE, FAKE, 0.1, FAKE, FAKE_ODD, None) == EALIGN
    assert lib.intsgd_decode_update(desc.ref(), None, FAKE, 0.1, FAKE, None, None) == EINVAL
    assert lib.intsgd_update_norm(desc.ref(), FAKE, FAKE, None, FAKE, need, None) == EINVAL
    assert lib.intsgd_update_norm(desc.ref(), FAKE, FAKE_ODD, FAKE, FAKE, need, None) == EALIGN
    assert lib.intsgd_update_norm(desc.ref(), FAKE, FAKE, FAKE, FAKE, 8, None) == EWORKSPACE
    assert lib.intsgd_compress_sum(desc.ref(), ptrs(4), FAKE, FAKE_ODD, FAKE, FAKE, need, None) == EALIGN
    assert lib.intsgd_compress_sum(desc.ref(), ptrs(4), None, FAKE, FAKE, FAKE, need, None) == EINVAL
    assert lib.intsgd_decode_update_norm(desc.ref(), FAKE, FAKE, 0.1, FAKE, FAKE, None, need, None) == EWORKSPACE
    assert lib.intsgd_decode_update_norm(desc.ref(), FAKE, FAKE, 0.0, FAKE, FAKE, FAKE, need, None) == EINVAL
    for beta, eps, eta in [(1.0, 1e-8, 0.1), (-0.1, 1e-8, 0.1), (0.9, -1.0, 0.1), (0.9, 1e-8, 0.0),
                           (float("nan"), 0.0, 0.1)]:
        assert lib.intsgd_next_alpha(desc.ref(), FAKE, FAKE, beta, eps, eta, FAKE, None) == EINVAL
    assert lib.intsgd_next_alpha(desc.ref(), None, FAKE, 0.9, 1e-8, 0.1, FAKE, None) == EINVAL


def test_launch_options_are_validated_per_descriptor():
    """Launch options travel with the descriptor of each call; the library keeps none."""
    ok = P.LaunchOpts(4096, 100, 4, 2)
    assert call_step_fused(P.Desc(1000, 4, opts=ok), ws=None) == EWORKSPACE     # passed validation
    for bad in ((1000, 0, 0), (512, 0, 0), (131072, 0, 0), (4097, 0, 0), (0, (1 << 20) + 1, 0),
                (0, 0, 1), (0, 0, 9), (0, 0, 0, 3)):
        desc = P.Desc(1000, 4, opts=P.LaunchOpts(*bad))
        assert call_step_fused(desc) == EINVAL, bad
        assert P.intsgd_workspace_bytes(desc) == 0
        assert lib.intsgd_prepare(desc.ref()) == EINVAL
    # profiling events: both or none
    for a, b, want in ((FAKE, None, EINVAL), (None, FAKE, EINVAL), (FAKE, FAKE, EWORKSPACE),
                       (None, None, EWORKSPACE)):
        desc = P.Desc(1000, 4, opts=P.LaunchOpts(start_event=a, stop_event=b))
        assert call_step_fused(desc, ws=None) == want
    # the workspace size does not depend on the options
    desc = P.Desc(10**7, 8)
    a = P.intsgd_workspace_bytes(desc)
    desc.opts = P.LaunchOpts(1024, 1 << 20, 8)
    assert P.intsgd_workspace_bytes(desc) == a
    desc.opts = None
    assert P.intsgd_workspace_bytes(desc) == a


def test_largest_sum_output_is_validated():
    """The optional per-block output of the descriptor: NULL or a 4-byte aligned device pointer."""
    desc = P.Desc(1000, 4)
    need = P.intsgd_workspace_bytes(desc)
    desc.c.largest_sum = FAKE + 2
    assert call_step_fused(desc) == EALIGN
    assert lib.intsgd_prepare(desc.ref()) == EALIGN
    assert P.intsgd_workspace_bytes(desc) == 0
    desc.c.largest_sum = FAKE + 4
    assert call_step_fused(desc, ws=None) == EWORKSPACE          # passed validation
    assert P.intsgd_workspace_bytes(desc) == need                # the size does not depend on it


def test_two_callers_hold_different_options():
    """No process-wide state: the same query answers per descriptor, in any interleaving."""
    big = 1 << 22
    auto = P.Desc(big, 2, rounding=P.ROUND_NEAREST_EVEN)
    tile = P.Desc(big, 2, rounding=P.ROUND_NEAREST_EVEN, opts=P.LaunchOpts(two_phase=1))
    phased = P.Desc(big, 8, rounding=P.ROUND_STOCHASTIC, opts=P.LaunchOpts(two_phase=2))
    for _ in range(3):
        assert P.intsgd_fused_step_form(auto) == 1
        assert P.intsgd_fused_step_form(tile) == 1
        assert P.intsgd_fused_step_form(phased) == 2
    assert not hasattr(lib, "intsgd_set_tuning") and not hasattr(lib, "intsgd_tap_next_launch")


def test_only_the_c_abi_is_exported():
    """The dynamic symbol table is the extern "C" names of include/intsgd.h and nothing else."""
    import shutil
    import subprocess
    nm = shutil.which("nm")
    if nm is None:
        pytest.skip("no nm")
    out = subprocess.check_output([nm, "-D", "--defined-only", binding.library_path()]).decode()
    names = sorted(line.split()[-1] for line in out.splitlines() if line.strip())
    assert names == declared_functions()


def test_whole_step_call_validation():
    desc = P.Desc(1000, 4)
    need = P.intsgd_workspace_bytes(desc)
    f = lib.intsgd_step_fused_next_alpha
    ok_args = lambda **kw: [kw.get("desc", desc.ref()), kw.get("g", ptrs(4)), kw.get("alpha", FAKE),
                            kw.get("eta", 0.1), kw.get("eta_next", 0.05), kw.get("x", FAKE),
                            kw.get("r", FAKE),
                            kw.get("beta", 0.9), kw.get("eps", 1e-8), kw.get("ns", FAKE),
                            kw.get("sat", FAKE), kw.get("ws", FAKE), kw.get("wb", need), None]
    assert f(*ok_args(r=None)) == EINVAL
    assert f(*ok_args(alpha=None)) == EINVAL
    assert f(*ok_args(beta=1.0)) == EINVAL
    assert f(*ok_args(eps=-1.0)) == EINVAL
    assert f(*ok_args(eta=0.0)) == EINVAL
    for eta_next in (0.0, -1.0, float("nan"), float("inf")):
        assert f(*ok_args(eta_next=eta_next)) == EINVAL
    assert f(*ok_args(x=FAKE_ODD)) == EALIGN
    assert f(*ok_args(wb=need - 1)) == EWORKSPACE
    assert f(*ok_args(desc=None)) == EINVAL


def test_static_scratch_call_validation():
    """The entry point that must not allocate: same checks, and a problem whose scratch need
    exceeds the static array is refused before any device call."""
    f = lib.intsgd_step_fused_static
    desc = P.Desc(1000, 4, rounding=P.ROUND_STOCHASTIC)
    args = lambda **kw: [kw.get("desc", desc.ref()), kw.get("g", ptrs(4)), kw.get("alpha", FAKE),
                         kw.get("eta", 0.1), kw.get("eta_next", 0.1), kw.get("x", FAKE),
                         kw.get("r", FAKE), kw.get("beta", 0.9), 1e-8, kw.get("ns", FAKE),
                         kw.get("sat", FAKE), None]
    assert f(*args(r=None)) == EINVAL
    assert f(*args(x=FAKE_ODD)) == EALIGN
    assert f(*args(eta_next=0.0)) == EINVAL
    assert f(*args(desc=None)) == EINVAL
    n = 128
    big = P.Desc(1 << 26, n, rounding=P.ROUND_STOCHASTIC, clip=1000, opts=P.LaunchOpts(tile_coords=1024))
    assert (12 + 8 * n) * ((1 << 26) // 1024) > P.STATIC_SCRATCH_BYTES
    a = args(desc=big.ref(), g=ptrs(n))
    assert f(*a) == EWORKSPACE


def test_momentum_calls_validation():
    desc = P.Desc(1000, 4)
    need = P.intsgd_workspace_bytes(desc)
    f = lib.intsgd_step_momentum
    args = lambda **kw: [desc.ref(), ptrs(4), FAKE, kw.get("eta", 0.1), kw.get("eta_next", 0.1),
                         kw.get("mu", 0.9), kw.get("wd", 1e-4), kw.get("x", FAKE), kw.get("m", FAKE),
                         kw.get("r", None), 0.9, 1e-8, FAKE, FAKE, FAKE, need, None]
    assert f(*args(m=None)) == EINVAL
    assert f(*args(m=FAKE_ODD)) == EALIGN
    for mu in (-0.1, 1.0, float("nan")):
        assert f(*args(mu=mu)) == EINVAL
    for wd in (-1e-4, float("inf"), float("nan")):
        assert f(*args(wd=wd)) == EINVAL
    assert f(*args(eta=0.0)) == EINVAL
    assert f(*args(r=FAKE, eta_next=0.0)) == EINVAL
    g = lib.intsgd_decode_update_momentum
    assert g(desc.ref(), FAKE, FAKE, 0.1, 0.9, 1e-4, FAKE, None, FAKE, FAKE, need, None) == EINVAL
    assert g(desc.ref(), FAKE, FAKE, 0.1, 1.5, 1e-4, FAKE, FAKE, FAKE, FAKE, need, None) == EINVAL
    assert g(desc.ref(), FAKE, FAKE, 0.1, 0.9, 1e-4, FAKE, FAKE, FAKE, None, need, None) == EWORKSPACE


def test_diana_call_validation():
    desc = P.Desc(1000, 4)
    need = P.intsgd_workspace_bytes(desc)
    f = lib.intsgd_diana_step
    args = lambda **kw: [desc.ref(), kw.get("g", ptrs(4)), kw.get("hl", ptrs(4)), kw.get("alpha", FAKE),
                         kw.get("eta", 0.1), kw.get("eta_next", 0.1), kw.get("x", FAKE),
                         kw.get("h", FAKE), kw.get("r", None), kw.get("beta", 0.0), 0.0, FAKE, FAKE,
                         FAKE, kw.get("wb", need), None]
    assert f(*args(hl=None)) == EINVAL
    assert f(*args(hl=ptrs(4, FAKE_ODD))) == EALIGN
    assert f(*args(h=None)) == EINVAL
    assert f(*args(h=FAKE_ODD)) == EALIGN
    assert f(*args(alpha=None)) == EINVAL
    assert f(*args(eta=-1.0)) == EINVAL
    assert f(*args(r=FAKE, beta=1.0)) == EINVAL
    assert f(*args(r=FAKE, eta_next=-0.1)) == EINVAL
    assert f(*args(wb=16)) == EWORKSPACE


def test_heuristic_alpha_validation():
    desc = P.Desc(1000, 4)
    need = P.intsgd_workspace_bytes(desc)
    f = lib.intsgd_heuristic_alpha
    assert f(desc.ref(), ptrs(4), 0, FAKE, FAKE, need, None) == ERANGE
    assert f(desc.ref(), ptrs(4), 32, FAKE, FAKE, need, None) == ERANGE
    assert f(desc.ref(), ptrs(4), 7, None, FAKE, need, None) == EINVAL
    assert f(desc.ref(), None, 7, FAKE, FAKE, need, None) == EINVAL
    assert f(desc.ref(), ptrs(4, FAKE_ODD), 7, FAKE, FAKE, need, None) == EALIGN
    assert f(desc.ref(), ptrs(4), 7, FAKE, None, need, None) == EWORKSPACE


def test_status_strings():
    for st in (0, -1, -2, -3, -4, -5, -6):
        assert P.intsgd_status_string(st) not in ("", "unknown status")
    assert P.intsgd_status_string(-99) == "unknown status"
    with pytest.raises(P.IntSGDError):
        P.intsgd_prepare(P.Desc(0, 1))


def test_host_alpha_rule_equals_the_oracle():
    """The library's host twin of a8 against the oracle's (Section 4.1 / Algorithm 2)."""
    rng = np.random.default_rng(2)
    for offsets in (None, [0, 3, 700, 701, 5000]):
        d, n = 5000, 6
        B = 1 if offsets is None else len(offsets) - 1
        off_np = None if offsets is None else np.array(offsets, np.uint64)
        desc = P.Desc(d, n, block_offsets=offsets)
        r = np.zeros(B)
        for k in range(5):
            ns = rng.uniform(1e-8, 1e-2, B)
            st, r_h, a_h = P.intsgd_next_alpha_host(desc, ns, r, 0.9, 1e-8, 0.1)
            r, ad, af, bad = oracle.next_alpha(ns, r, d=d, n=n, beta=0.9, eps=1e-8, eta=0.1,
                                               offsets=off_np)
            assert st == 0 and bad == 0
            assert np.array_equal(np.array(r_h), r)
            assert np.array_equal(np.array(a_h, np.float32), af)
    st, _, a = P.intsgd_next_alpha_host(P.Desc(10, 1), [0.0], [0.0], 0.0, 0.0, 0.1)
    assert st == ERANGE and np.isposinf(a[0])


def test_fused_step_form_policy():
    """Host-only query of which sweep the fused step would launch."""
    big, small = 1 << 22, (1 << 22) - 1
    four = P.LaunchOpts(two_phase=2)
    assert P.intsgd_fused_step_form(P.Desc(big, 4, rounding=P.ROUND_NEAREST_EVEN, opts=four)) == 2
    assert P.intsgd_fused_step_form(P.Desc(small, 4, rounding=P.ROUND_NEAREST_EVEN, opts=four)) == 1
    assert P.intsgd_fused_step_form(P.Desc(big, 8, rounding=P.ROUND_STOCHASTIC)) == 1
    blocks = P.Desc(big, 8, rounding=P.ROUND_NEAREST_EVEN, block_offsets=[0, 1000, big])
    assert P.intsgd_fused_step_form(blocks) == 1
    for n, form in [(1, 1), (2, 1), (5, 1), (8, 1), (16, 1), (128, 1)]:       # automatic: the tile sweep
        assert P.intsgd_fused_step_form(P.Desc(big, n, rounding=P.ROUND_NEAREST_EVEN)) == form
    two = P.LaunchOpts(two_phase=2)
    assert P.intsgd_fused_step_form(P.Desc(big, 8, rounding=P.ROUND_STOCHASTIC, opts=two)) == 2
    blocks.opts = two
    assert P.intsgd_fused_step_form(blocks) == 1
    assert P.intsgd_fused_step_form(P.Desc(small, 8, opts=two)) == 1
    one = P.LaunchOpts(two_phase=1)
    assert P.intsgd_fused_step_form(P.Desc(big, 2, rounding=P.ROUND_NEAREST_EVEN, opts=one)) == 1
    assert lib.intsgd_fused_step_form(None) == 0


def test_traffic_table_keys_match_workload_names():
    """bench.py looks HBM traffic up by "<workload name>/<sweep form>"; the committed table
    must use names the workload recipes really have."""
    import json
    import os

    from paper_2102_08374_amd import workloads as W
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles",
                        "traffic.json")
    with open(path) as fh:
        table = json.load(fh)
    names = {W.config(i, rounding=r).name for i in range(1, 6) for r in (None, 0, 1)}
    names.add(W.config(4, per_bucket=False).name)
    keys = [k for k in table if not k.startswith("_")]
    assert keys, "empty traffic table"
    for k in keys:
        name, form = k.rsplit("/", 1)
        assert name in names, k
        assert form in ("tile", "two_phase"), k
        assert table[k]["bytes_per_launch"] == table[k]["fetch_bytes"] + table[k]["write_bytes"]
    # the headline workload has the entry bench.py reports by default
    assert W.config(5).name + "/tile" in table


def test_header_is_plain_c_and_links(tmp_path):
    """include/intsgd.h compiles as C99 (-pedantic, warnings as errors) and a C program
    linked against the built library can call the host-only entry points."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "abi.c"
    src.write_text(
        '#include "intsgd.h"\n#include <stdio.h>\n#include <string.h>\n'
        "int main(void) {\n"
        "  intsgd_desc d; double nsq = 1e-6, r = 0.0; float a = 0.0f; intsgd_status st;\n"
        "  memset(&d, 0, sizeof d);\n"
        "  if (intsgd_workspace_bytes(&d) != 0) return 2;\n"
        "  d.d = 1048576; d.n = 4; d.num_blocks = 1; d.rounding = INTSGD_ROUND_STOCHASTIC;\n"
        "  d.wire = INTSGD_WIRE_INT32; d.clip = 536870911;\n"
        "  if (intsgd_workspace_bytes(&d) == 0) return 3;\n"
        "  st = intsgd_next_alpha_host(&d, &nsq, &r, 0.9, 1e-8, 0.1, &a);\n"
        '  printf("%d %.9g %s\\n", (int)st, (double)a, intsgd_status_string(INTSGD_EALIGN));\n'
        "  return 0;\n}\n")
    exe = tmp_path / "abi"
    libdir = os.path.dirname(binding.library_path())
    subprocess.check_call([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                           "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                           "-L", libdir, "-lintsgd", "-lm", "-Wl,-rpath," + libdir])
    out = subprocess.check_output([str(exe)]).decode().split(None, 2)
    assert out[0] == "0"
    w = oracle.next_alpha(np.array([1e-6]), np.array([0.0]), n=4, d=1048576, beta=0.9, eps=1e-8, eta=0.1)
    assert np.float32(float(out[1])) == np.float32(w[1][0])
    assert out[2].strip() == "vector pointer not 16-byte aligned"
