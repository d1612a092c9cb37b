"""Host-side checks that need no GPU: the shared library loads, exports what include/corey.h declares,
rejects bad arguments before launching anything, and its chunk rule agrees with the oracle's."""
import ctypes
import math
import os
import re

import pytest

import oracle
from conftest import ROOT, read_golden
from paper_2604_10597_amd import binding


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "corey.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(corey_\w+|selective_scan_fwd\w*|causal_conv1d_silu_fwd|selective_state_update)\s*\(", hdr))
    declared -= {"corey_dtype", "corey_status", "corey_policy"}
    assert declared == set(binding.EXPORTS)
    lib = binding.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert binding.corey_version() == "0.1"


def test_binding_constants_are_the_headers():
    """The numbers the Python binding carries (it cannot include the header) against include/corey.h."""
    hdr = open(os.path.join(ROOT, "include", "corey.h")).read()
    defs = dict(re.findall(r"^#define\s+(COREY_\w+)\s+(.+?)\s*(?:/\*.*)?$", hdr, flags=re.M))
    val = lambda name: eval(re.sub(r"(\d)u\b", r"\1", re.sub(r"COREY_\w+", lambda m: "(" + defs[m.group(0)] + ")", defs[name])))
    assert binding.HANDOFF_BYTES == val("COREY_HANDOFF_BYTES") and binding.CHUNK_SLOTS == val("COREY_CHUNK_SLOTS")
    assert binding.COREY_SCAN_GENERAL_A == val("COREY_SCAN_GENERAL_A") and binding.COREY_SCAN_ONE_CHUNK == val("COREY_SCAN_ONE_CHUNK")
    assert binding.COREY_SCAN_WHOLE_ROWS == val("COREY_SCAN_WHOLE_ROWS")
    enum = re.search(r"typedef enum \{([^}]*)\} corey_dtype;", hdr).group(1)
    codes = {k: int(v) for k, v in re.findall(r"(COREY_(?:F32|BF16|F16))\s*=\s*(\d+)", enum)}
    assert (binding.COREY_F32, binding.COREY_BF16, binding.COREY_F16) == (codes["COREY_F32"], codes["COREY_BF16"], codes["COREY_F16"])


def _href(tok):
    return math.log(int(tok.split(":")[1])) if tok.startswith("logK:") else float(tok)


@pytest.mark.parametrize("row", read_golden("chunk_rule_pins.txt"), ids=lambda r: "-".join(r))
def test_library_chunk_rule_on_the_papers_values(row):
    H, href, cmin, cmax, expect = float(row[0]), _href(row[1]), int(row[2]), int(row[3]), int(row[4])
    p = binding.policy_default()
    p.c_min, p.c_max = cmin, cmax
    assert binding.corey_select_chunk(min(H / href, 1.0), 4096, p) == expect


def test_library_chunk_rule_matches_oracle_everywhere():
    for mode in (0, 1, 2, 3, 4):
        for cmin, cmax in ((64, 2048), (32, 512), (128, 128)):
            p = binding.policy_default()
            p.mode, p.c_min, p.c_max = mode, cmin, cmax
            op = oracle.policy(mode=mode, c_min=cmin, c_max=cmax)
            for scale in (1.0, math.log(256) / 8.0):
                p.h_ref_scale = op.h_ref_scale = scale
                for L in (1, 25, 50, 51, 256, 300, 4096, 16384):
                    for i in range(0, 201):
                        r = i / 200.0
                        st, c, margin = oracle.select_chunk(r, L, op)
                        assert st == oracle.OK
                        assert binding.corey_select_chunk(r, L, p) == c, (mode, cmin, cmax, L, r, margin)


def test_chunk_rule_errors():
    p = binding.policy_default()
    with pytest.raises(binding.CoreyError) as e:
        binding.corey_select_chunk(float("nan"), 4096, p)
    assert e.value.code == 4
    with pytest.raises(binding.CoreyError) as e:
        binding.corey_select_chunk(0.5, 0, p)
    assert e.value.code == 1
    p.c_min = 48
    with pytest.raises(binding.CoreyError):
        binding.corey_select_chunk(0.5, 64, p)
    p = binding.policy_default()
    p.mode = 9
    with pytest.raises(binding.CoreyError):
        binding.corey_select_chunk(0.5, 64, p)
    assert binding.lib().corey_select_chunk(0.5, 64, None, None) == 2
    assert b"NULL" in binding.lib().corey_last_error()


def test_gpu_entry_points_reject_bad_arguments_before_any_launch():
    lib = binding.lib()
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: every call below fails validation first
    none = ctypes.c_void_p(0)
    eh = lambda **kw: lib.corey_entropy_hist(
        kw.get("x", fake), kw.get("dt", 1), kw.get("B", 1), kw.get("D", 4), kw.get("L", 8), kw.get("seqlens", none), kw.get("K", 16),
        kw.get("eps", 1e-8), kw.get("stride", 1), kw.get("block", 1), kw.get("counts", fake), fake, fake, none, kw.get("rp", none),
        kw.get("ws", fake), kw.get("wsb", 256), none)
    assert eh(x=none) == 2 and eh(counts=none) == 2
    assert eh(dt=7) == 1 and eh(K=1) == 1 and eh(K=5000) == 1 and eh(stride=0) == 1 and eh(block=0) == 1 and eh(eps=-1.0) == 1
    assert eh(B=0) == 3 and eh(L=0) == 3
    assert eh(ws=none) == 7 and eh(wsb=8) == 7
    assert eh(rp=fake, seqlens=fake) == 1 and eh(rp=ctypes.c_void_p(0x1004)) == 1     # given range: whole tensor only, aligned

    cv = lambda **kw: lib.causal_conv1d_silu_fwd(
        kw.get("x", fake), kw.get("w", fake), none, none, kw.get("u", ctypes.c_void_p(0x2000)), none, kw.get("rp", none),
        kw.get("pt", none), kw.get("ptb", 0), kw.get("dt", 1), kw.get("B", 1), kw.get("D", 4), kw.get("L", 8), kw.get("W", 4), none)
    big = lib.corey_pattern_table_workspace()
    assert big > 256 * 131072
    assert cv(pt=fake, ptb=big, dt=0) == 5 and cv(pt=fake, ptb=1024) == 7 and cv(pt=ctypes.c_void_p(0x1010), ptb=big) == 7
    assert cv(x=none) == 2 and cv(w=none) == 2 and cv(u=none) == 2
    assert cv(dt=9) == 1 and cv(W=0) == 1 and cv(W=5) == 1 and cv(u=fake) == 1 and cv(rp=ctypes.c_void_p(0x1004)) == 1
    assert cv(B=0) == 3 and cv(L=0) == 3
    assert lib.corey_entropy_hist_workspace(0, 16) == 0 and lib.corey_entropy_hist_workspace(3, 1) == 0
    assert lib.corey_entropy_hist_workspace(3, 256) >= 3 * 16

    one = lambda **kw: lib.corey_entropy_hist_onesweep(
        kw.get("x", fake), kw.get("dt", 1), kw.get("B", 1), kw.get("D", 4), kw.get("L", 8), kw.get("K", 16), kw.get("eps", 1e-8),
        kw.get("p", None), kw.get("chunks", none), kw.get("counts", fake), fake, fake, none, kw.get("ws", fake), kw.get("wsb", big), none)
    assert one(x=none) == 2 and one(counts=none) == 2 and one(dt=0) == 5 and one(dt=9) == 1 and one(K=1) == 1 and one(eps=-1.0) == 1
    assert one(B=0) == 3 and one(B=1 << 20, D=1 << 10, L=1 << 10) == 3 and one(ws=none) == 7 and one(wsb=4096) == 7
    assert one(x=ctypes.c_void_p(0x1001)) == 1 and one(p=ctypes.byref(binding.policy_default())) == 2     # a policy needs chunks_out
    ft = lambda **kw: lib.corey_entropy_hist_from_table(kw.get("dt", 1), kw.get("L", 8), kw.get("K", 16), 1e-8, None, none,
                                                        kw.get("counts", fake), fake, fake, none, kw.get("ws", fake), kw.get("wsb", big), none)
    assert ft(counts=none) == 2 and ft(dt=0) == 5 and ft(K=5000) == 1 and ft(L=0) == 3 and ft(ws=none) == 7 and ft(wsb=1) == 7

    su = lambda **kw: lib.selective_state_update(
        kw.get("state", fake), kw.get("x", fake), fake, fake, fake, fake, none, none, none, 1, kw.get("y", fake), kw.get("dt", 1),
        kw.get("B", 1), kw.get("D", 4), kw.get("N", 16), none)
    assert su(state=none) == 2 and su(x=none) == 2 and su(y=none) == 2
    assert su(dt=5) == 1 and su(state=ctypes.c_void_p(0x1002)) == 1
    assert su(B=0) == 3 and su(N=0) == 3 and su(N=257) == 3 and su(B=1 << 20, D=1 << 10) == 3

    ss = lambda **kw: lib.selective_scan_fwd(
        kw.get("u", fake), fake, fake, fake, fake, none, none, none, 1, none, none, kw.get("chunk", 256), none,
        kw.get("y", fake), kw.get("last", fake), kw.get("dt", 1), kw.get("B", 1), kw.get("D", 4), kw.get("N", 16),
        kw.get("L", 64), kw.get("flags", 0), kw.get("ws", fake), kw.get("wsb", 1 << 30), none)
    assert ss(u=none) == 2 and ss(y=none) == 2 and ss(last=none) == 2
    assert ss(dt=3) == 1 and ss(flags=8) == 1 and ss(flags=0x80000001) == 1
    for bad in (0, 8, 100, 4096, -64):
        assert ss(chunk=bad) == 1
    assert ss(N=0) == 3 and ss(N=257) == 3 and ss(B=0) == 3 and ss(L=0) == 3 and ss(B=70000) == 3
    assert ss(ws=none) == 7 and ss(wsb=64) == 7
    assert lib.selective_scan_fwd_workspace(1, 16, 64) == 4 * 16 * (64 + 2048) * 4
    assert lib.selective_scan_fwd_workspace(0, 16, 64) == 0 and lib.selective_scan_fwd_workspace(1, 300, 64) == 0


def test_device_rule_rejects_a_policy_that_can_pick_a_chunk_the_scan_cannot_run():
    """corey_select_chunk_device / corey_route_device feed selective_scan_fwd's chunks_dev and the chunk-distribution
    counters (one slot per power of two up to COREY_MAX_CHUNK): a policy that can select more is refused on the host."""
    lib = binding.lib()
    fake, none = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    for field, mode in (("c_max", 0), ("c_max", 1), ("c_max", 4), ("static_chunk", 3), ("long_chunk", 2), ("short_chunk", 2),
                        ("short_chunk", 1), ("safe_chunk", 4)):
        p = binding.policy_default()
        p.mode = mode
        setattr(p, field, 4096)
        assert lib.corey_select_chunk_device(fake, none, 4096, 1, ctypes.byref(p), fake, none) == 1, (field, mode)
        assert lib.corey_route_device(fake, 1, 1, 4, 8, none, 16, 1e-8, 1, 1, ctypes.byref(p), 0.0, none, none, fake, fake, fake, none,
                                      none, fake, fake, 1 << 20, none) == 1, (field, mode)
        assert binding.corey_select_chunk(0.99, 1 << 20, p) > 0            # the host rule itself has no such limit
    p = binding.policy_default()
    p.static_chunk = 4096                                                  # unused by the mode: accepted
    assert lib.corey_select_chunk_device(none, none, 4096, 1, ctypes.byref(p), fake, none) == 2   # (fails later, on the NULL r)


def test_launch_plan_of_the_scan():
    """Host logic of the scan's launch shape: which leading channels take 16 time steps per lane."""
    plan = binding.selective_scan_fwd_plan
    assert plan(0, 64, 16, 256) == -1 and plan(1, 64, 16, 100) == -1 and plan(1, 64, 300, 256) == -1
    # every row can have a resident wave of its own: all rows with 8 steps per lane
    assert plan(1, 64, 16, 256) == 0 and plan(1, 4096, 16, 512) == 0 and plan(1, 5120, 16, 256) == 0
    # beyond that: whole layers of one workgroup per compute unit with 16 steps, the remainder with 8
    assert plan(1, 5120, 16, 512) == 4096 and plan(1, 7168, 16, 512) == 6144 and plan(1, 6144, 16, 512) == 6144
    assert plan(2, 2100, 16, 512) == 2048 and plan(1, 12288, 16, 256) == 12288 and plan(1, 10240, 16, 256) == 8192
    # a row of 8-step lanes no longer fits a wave above chunk 512
    assert plan(1, 64, 16, 1024) == 64 and plan(4, 2048, 16, 2048) == 2048
    for B in (1, 2, 3, 5, 8):
        for D in (1, 31, 32, 100, 1536, 4097, 5120, 9000, 40000):
            for N in (1, 16, 64, 256):
                for chunk in (16, 64, 128, 256, 512, 1024, 2048):
                    d16 = plan(B, D, N, chunk)
                    assert 0 <= d16 <= D and (d16 == D or d16 % 32 == 0), (B, D, N, chunk, d16)
                    steps = binding.selective_scan_fwd_plan_steps(B, D, N, chunk)
                    assert steps in (4, 8) and (steps == 8 or (d16 == 0 and chunk <= 256)), (B, D, N, chunk, d16, steps)
    # launches of one geometry with at most 1536 waves give a channel two rows (tiles up to 1024 steps, N >= 4)
    split = binding.selective_scan_fwd_plan_split
    assert split(0, 64, 16, 256) == -1 and split(1, 64, 16, 100) == -1
    assert split(1, 64, 16, 256) == 1 and split(1, 64, 16, 1024) == 1 and split(1, 64, 16, 2048) == 0 and split(1, 64, 3, 256) == 0
    assert split(1, 1024, 16, 1024) == 1 and split(1, 1536, 16, 1024) == 1 and split(1, 1537, 16, 1024) == 0     # 64 lanes per row
    assert split(1, 1536, 16, 512) == 1 and split(1, 5120, 16, 512) == 0 and split(1, 5120, 16, 128) == 0
    assert split(1, 5120, 16, 64) == 1 and split(1, 5120, 16, 16) == 1 and split(4, 2048, 16, 32) == 1 and split(4, 2048, 16, 64) == 0
    # short of waves (few channels or short tiles, a 4-step row still inside one wave): 4 steps per lane
    steps = binding.selective_scan_fwd_plan_steps
    assert steps(0, 64, 16, 256) == -1 and steps(1, 64, 16, 100) == -1
    assert steps(1, 1536, 16, 256) == 4 and steps(1, 1536, 16, 512) == 8 and steps(1, 5120, 16, 128) == 4
    assert steps(1, 5120, 16, 256) == 8 and steps(4, 2048, 16, 64) == 4 and steps(4, 2048, 16, 128) == 8
    assert steps(1, 13000, 16, 64) == 8 and plan(1, 13000, 16, 64) == 0 and steps(1, 50000, 16, 16) == 8


def test_product_fails_loudly_without_the_library_and_never_reaches_for_the_oracle():
    """No CPU fallback: with the shared library missing the package raises on first use, and nothing under the product
    package imports the oracle."""
    import subprocess
    import sys
    code = ("import paper_2604_10597_amd as c, sys\n"
            "try:\n    c.corey_version()\nexcept Exception as e:\n    print(type(e).__name__, e); sys.exit(7)\n")
    env = dict(os.environ, COREY_LIB="/nonexistent/libcorey.so", PYTHONPATH=ROOT)
    r = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 7 and "libcorey" in r.stdout, (r.returncode, r.stdout, r.stderr)
    pkg = os.path.join(ROOT, "paper_2604_10597_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "corey_oracle" not in text, f


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
