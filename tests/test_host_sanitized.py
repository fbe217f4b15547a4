"""The library's host-side arithmetic (routing, plan validation / prefix sums /
chunk geometry, batch alias sweep and staging size, goodput planner) compiled
for the CPU alone with AddressSanitizer and UndefinedBehaviorSanitizer and
driven through tests/host_sanitize/host_check.cpp.  Results are compared with
the oracle (route, planner) or with arithmetic written out here (geometry,
overlap by brute force); any sanitizer report makes the driver exit non-zero."""
import itertools
import os
import subprocess

import numpy as np
import pytest

from oracle import kvmig as orc
from oracle import planner as op
from workload import SplitMix64
from workload.planner import synthetic_tiers

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_05467_amd", "csrc")
HERE = os.path.join(ROOT, "tests", "host_sanitize")
EXE = os.path.join(HERE, "host_check_san")


@pytest.fixture(scope="module")
def run():
    srcs = [os.path.join(HERE, "host_check.cpp"), os.path.join(CSRC, "nts_host.hip"), os.path.join(CSRC, "nts_planner.hip")]
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-Wall", "-Wextra",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-x", "c++"] + srcs + ["-o", EXE]
    subprocess.check_call(cmd)

    def feed(lines):
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        p = subprocess.run([EXE], input="\n".join(lines) + "\n", capture_output=True, text=True, env=env)
        assert p.returncode == 0 and p.stderr == "", p.stderr[-3000:]
        out = p.stdout.splitlines()
        assert len(out) == len(lines)
        return [l.split() for l in out]

    return feed


def test_route_everywhere(run):
    cases = [(H, Ns, rs, Nd, rd) for H in (8, 16, 32, 64) for Ns in (1, 2, 4, 8) for Nd in (1, 2, 4, 8)
             for rs in range(Ns) for rd in range(Nd)]
    bad = [(8, 3, 0, 1, 0), (8, 2, 2, 1, 0), (8, 1, 0, 16, 0), (0, 1, 0, 1, 0), (8, 2, -1, 2, 0),
           (2 ** 31 - 1, 1, 0, 1, 0), (-8, 2, 0, 2, 0)]
    out = run(["route %d %d %d %d %d" % c for c in cases + bad])
    for c, o in zip(cases, out):
        assert [int(x) for x in o[1:]] == [0, *orc.route(*c)], c
    for c, o in zip(bad[:5], out[len(cases):]):
        assert int(o[1]) == -1, c
    assert int(out[-2][1]) == 0 and int(out[-1][1]) == -1
    # a single head, and a result pointer missing
    assert [int(x) for x in run(["route 1 1 0 1 0"])[0][1:]] == [0, 0, 0, 1]
    assert [int(o[1]) for o in run(["route_null %d" % k for k in range(3)])] == [-1, -1, -1]


def _geom_line(L, D, e, p, Hs, Hd, so, do, w, S_src, S_dst, sst, dst, staging, lens):
    return "geom %d %d %d %d %d %d %d %d %d %d %d %d %d %d 1 %d %s" % (
        L, D, e, p, Hs, Hd, so, do, w, S_src, S_dst, sst, dst, staging, len(lens), " ".join(str(int(x)) for x in lens))


def test_plan_geometry_against_written_out_arithmetic(run):
    rng = SplitMix64(31)
    u = lambda lo, hi: int(rng.integers(lo, hi, 1)[0])
    cases = []
    for i in range(300):
        e = (1, 2, 4)[u(0, 2)]
        D = (3, 8, 24, 64, 128, 100)[u(0, 5)]
        Hs, Hd = u(1, 8), u(1, 8)
        w = u(1, min(Hs, Hd))
        so, do = u(0, Hs - w), u(0, Hd - w)
        p = (1, 1, 2, 16)[u(0, 3)]
        L = u(1, 96)
        n_req = u(0, 12)
        lens = rng.integers(0, 3000, n_req) if n_req else np.zeros(0, np.int64)
        pad_s, pad_d = (0, 0, 4, 16)[u(0, 3)], (0, 8, 0, 32)[u(0, 3)]
        sst = 0 if pad_s == 0 and u(0, 1) else Hs * D * e + pad_s
        dstr = 0 if pad_d == 0 and u(0, 1) else Hd * D * e + pad_d
        staging = (0, 1, 777, 65536, 1 << 20, 64 << 20, 1 << 40)[u(0, 6)]
        cases.append((L, D, e, p, Hs, Hd, so, do, w, 4096 * p, 8192 * p, sst, dstr, staging, lens))
    # the headline shapes: 4096 tokens <-> 2^29 bytes, 720896 tokens in 1409 chunks of 64 MiB
    cases.append((32, 128, 2, 1, 8, 8, 0, 0, 8, 49152, 49152, 0, 0, 0, [4096]))
    cases.append((32, 128, 2, 1, 8, 8, 0, 0, 8, 753664, 753664, 0, 0, 0, [720896]))
    cases.append((96, 1 << 20, 4, 1, 1, 1, 0, 0, 1, 1 << 30, 1 << 30, 0, 0, 1 << 62, [2 ** 31 - 1]))   # widest legal numbers
    out = run([_geom_line(*c) for c in cases])
    for c, o in zip(cases, out):
        L, D, e, p, Hs, Hd, so, do, w, S_src, S_dst, sst, dstr, staging, lens = c
        frag = w * D * e
        ss, ds = sst or Hs * D * e, dstr or Hd * D * e
        vec = next((v for v in (16, 8, 4) if all(x % v == 0 for x in (frag, ss, ds, so * D * e, do * D * e))), 0)
        if vec == 0:
            assert int(o[1]) == -1, c
            continue
        assert int(o[1]) == 0, (c, o)
        lens = np.asarray(lens, np.int64)
        T, NP = int(lens.sum()), int(((lens + p - 1) // p).sum())
        F = T * 2 * L
        cf = max(1, (staging or 64 << 20) // frag)
        cf_max = ((2 ** 31 - 64) // (frag // vec)) // 2
        cf = min(cf, max(cf_max, 1))
        n_chunks = -(-F // cf)
        got = [int(x) for x in o[2:13]]
        assert got == [T, NP, F, frag, F * frag, cf, cf * frag, n_chunks, ss, ds, vec], (c, got)
        n = len(lens)
        offs = [int(x) for x in o[13:13 + 2 * (n + 1)]]
        assert offs[:n + 1] == [0, *np.cumsum(lens).tolist()]
        assert offs[n + 1:] == [0, *np.cumsum((lens + p - 1) // p).tolist()]
        assert o[-2:] == ["tiles", "1"]
    assert [int(x) for x in out[-3][2:10]] == [4096, 4096, 262144, 2048, 2 ** 29, 32768, 64 << 20, 8]
    assert int(out[-2][9]) == 1408          # 88 GiB in 64 MiB chunks


def test_plan_geometry_rejections(run):
    ok = dict(L=2, D=64, e=2, p=1, Hs=4, Hd=4, so=0, do=0, w=4, S_src=64, S_dst=64, sst=0, dst=0, staging=0, lens=[3, 4])
    bad = [dict(L=0), dict(L=97), dict(D=0), dict(D=(1 << 20) + 1), dict(e=3), dict(p=0), dict(Hs=0), dict(Hd=70000),
           dict(w=0), dict(w=5), dict(so=1), dict(do=-1), dict(so=2 ** 31 - 1), dict(S_src=0), dict(S_dst=2 ** 31),
           dict(p=2, S_src=63), dict(sst=500), dict(dst=(1 << 30) + 4), dict(D=1, e=1, w=3), dict(lens=[3, -1]),
           dict(lens=[2 ** 31 - 1, 1]),
           # each side by itself: a bad value on one side with a good one on the other
           dict(so=-1), dict(do=1), dict(Hs=8, so=5), dict(Hd=8, do=5), dict(Hs=70000), dict(Hd=0),
           dict(S_dst=0), dict(S_src=2 ** 31), dict(p=2, S_dst=63), dict(dst=500), dict(sst=(1 << 30) + 4)]
    # ... and the last value each of those checks lets through
    good = [dict(L=1), dict(L=96), dict(D=1, e=4), dict(D=1 << 20, sst=1 << 30, dst=1 << 30, Hs=64, Hd=64),
            dict(Hs=8, so=4), dict(Hd=8, do=4), dict(Hs=65536, Hd=65536, D=2), dict(S_src=1, S_dst=1),
            dict(S_src=2 ** 31 - 1, S_dst=2 ** 31 - 1), dict(sst=1 << 30), dict(dst=1 << 30), dict(lens=[2 ** 31 - 1]),
            dict(lens=[]), dict(lens=[0, 0])]
    lines = []
    for o in bad:
        c = dict(ok, **o)
        lines.append(_geom_line(c["L"], c["D"], c["e"], c["p"], c["Hs"], c["Hd"], c["so"], c["do"], c["w"], c["S_src"],
                                c["S_dst"], c["sst"], c["dst"], c["staging"], c["lens"]))
    out = run(lines + [_geom_line(*[ok[k] for k in ("L", "D", "e", "p", "Hs", "Hd", "so", "do", "w", "S_src", "S_dst",
                                                     "sst", "dst", "staging", "lens")])])
    for o, b in zip(out[:-1], bad):
        assert int(o[1]) == -1, (b, o)
    assert int(out[-1][1]) == 0
    keys = ("L", "D", "e", "p", "Hs", "Hd", "so", "do", "w", "S_src", "S_dst", "sst", "dst", "staging", "lens")
    for o, g in zip(run([_geom_line(*[dict(ok, **g)[k] for k in keys]) for g in good]), good):
        assert int(o[1]) == 0, (g, o)
    # a page table may be missing only when there is no token to look up
    line = _geom_line(*[ok[k] for k in keys])
    empty = _geom_line(*[dict(ok, lens=[0, 0])[k] for k in keys])
    out = run([line.replace("geom", v, 1) for v in ("geom_nosrc", "geom_nodst")] +
              [empty.replace("geom", v, 1) for v in ("geom_nosrc", "geom_nodst")])
    assert [int(o[1]) for o in out] == [-1, -1, 0, 0]
    single = _geom_line(*[dict(ok, lens=[0, 1])[k] for k in keys])              # one token is enough to need them
    assert [int(o[1]) for o in run([single.replace("geom", v, 1) for v in ("geom_nosrc", "geom_nodst", "geom")])] == [-1, -1, 0]


def test_alias_sweep_against_brute_force(run):
    rng = SplitMix64(8)
    u = lambda lo, hi: int(rng.integers(lo, hi, 1)[0])
    cases, lines = [], []
    for i in range(400):
        n = u(0, 10)
        base = u(1, 2 ** 40)
        rs = []
        for _ in range(n):
            lo = base + u(0, 4000)
            rs.append((lo, lo + u(1, 600), u(0, 1)))
        stg, sb = base + u(0, 6000), u(1, 500)
        cases.append((rs, stg, sb))
        lines.append("alias %d %s %d %d" % (n, " ".join("%d %d %d" % r for r in rs), stg, sb))
    # ranges that end at the top of the address space
    top = 2 ** 64 - 1
    cases.append(([(top - 100, top, 0), (top - 300, top - 100, 1)], 4096, 64))
    lines.append("alias 2 %d %d 0 %d %d 1 4096 64" % (top - 100, top, top - 300, top - 100))
    # ranges that only touch: a pool ending where the staging area or a pool of the other side begins
    for rs, stg, sb in [([(1000, 2000, 0)], 2000, 100), ([(1000, 2000, 1)], 900, 100), ([(1000, 2000, 0)], 1999, 2),
                        ([(1000, 2000, 0)], 999, 2), ([(1000, 2000, 0), (2000, 3000, 1)], 5000, 16),
                        ([(2000, 3000, 0), (1000, 2000, 1)], 5000, 16), ([(1000, 2001, 0), (2000, 3000, 1)], 5000, 16)]:
        cases.append((rs, stg, sb))
        lines.append("alias %d %s %d %d" % (len(rs), " ".join("%d %d %d" % r for r in rs), stg, sb))
    out = run(lines)
    seen = set()
    for (rs, stg, sb), o in zip(cases, out):
        hit = lambda a, b: a[0] < b[1] and b[0] < a[1]
        want = any(hit(a, b) for a, b in itertools.combinations(rs, 2) if a[2] != b[2]) or \
            any(hit(a, (stg, stg + sb)) for a in rs)
        assert int(o[1]) == (-4 if want else 0), (rs, stg, sb)
        seen.add(want)
    assert seen == {True, False}
    out = run(["staging 0", "staging 3 60 64 17", "staging 1 67108860", "staging 2 %d 16" % (2 ** 40)])
    assert [int(o[1]) for o in out] == [0, 128, 2 * 67108864, 2 ** 41]


def test_planner_matches_the_oracle(run):
    lines, want = [], []
    for thp, thd in itertools.product([1.0, 2.5, 3.0, 7.0, 10.0, 13.7], repeat=2):
        for m in (1, 4, 8):
            lines.append("block %r %r %d" % (thp, thd, m))
            want.append(["block", "0", *map(str, op.balanced_block(thp, thd, m))])
        P, D = op.balanced_block(thp, thd)
        for rps in (0.5, 5.0, 1e6):
            lines.append("ge %r 2 %r 4 %d %d %r" % (thp, thd, P, D, rps))
            want.append(["ge", "0", repr(op.goodput_efficiency(thp, 2, thd, 4, P, D, rps))])
    out = run(lines)
    for o, w in zip(out, want):
        assert o[:2] == w[:2] and ([float(x) for x in o[2:]] == [float(x) for x in w[2:]]), (o, w)
    lines, want = [], []
    for seed in range(10):
        tiers = synthetic_tiers(seed, 1 + seed % 5)
        for G in (0, 3, 8, 16, 64, 128, 1024):
            lines.append("plan %d %d 8 4096 %s" % (G, len(tiers), " ".join(
                "%r %s %s" % (float(t[0]), " ".join(repr(float(x)) for x in t[1]), " ".join(repr(float(x)) for x in t[2]))
                for t in tiers)))
            want.append(op.plan(G, [op.Tier(*t) for t in tiers]))
    from planner_cases import INSTANCES, INVALID_TIERS
    fmt = lambda tiers: " ".join(
        "%r %s %s" % (float(t[0]), " ".join(repr(float(x)) for x in t[1]), " ".join(repr(float(x)) for x in t[2])) for t in tiers)
    for G, tiers in INSTANCES:
        lines.append("plan %d %d 8 4096 %s" % (G, len(tiers), fmt(tiers)))
        want.append(op.plan(G, [op.Tier(*t) for t in tiers]))
    bad = run(["plan 8 %d 8 64 %s" % (len(t), fmt(t)) for t in INVALID_TIERS] +
              ["block 0.0 1.0 8", "block 1.0 0.0 8", "block -1.0 1.0 8", "block nan 1.0 8", "block 1.0 1.0 0",
               "ge 0.0 1 1.0 1 1 1 1.0", "ge 1.0 1 0.0 1 1 1 1.0", "ge 1.0 0 1.0 1 1 1 1.0", "ge 1.0 1 1.0 0 1 1 1.0",
               "ge 1.0 1 1.0 1 0 1 1.0", "ge 1.0 1 1.0 1 1 0 1.0", "ge 1.0 1 1.0 1 1 1 -1.0", "plan 8 1 0 64 5.0 1 1 1 1 1 1 1 1",
               "plan -1 1 8 64 5.0 1 1 1 1 1 1 1 1"])
    assert all(int(o[1]) == -1 for o in bad), bad
    assert run(["ge 1.0 1 1.0 1 1 1 0.0"])[0][1:] == ["0", "0"]
    # legal corner cases: no tier at all, a tier that asks for nothing, one instance per side, no room asked for
    # in the output array when no step is taken
    one = "5.0 1 1 1 1 1 1 1 1"
    corner = run(["plan 8 0 8 4", "plan 8 1 8 4 0.0 1 1 1 1 1 1 1 1", "plan 8 1 1 64 " + one, "plan 0 1 8 0 " + one,
                  "plan 1 1 8 0 " + one])
    assert corner[0][1:4] == ["0", "0", "8"] and corner[1][1:4] == ["0", "0", "8"]
    assert corner[2][1:3] == ["0", "4"] and corner[2][3] == "0"           # four blocks of 1 + 1 GPUs serve 4 of the 5 req/s
    assert corner[3][1:4] == ["0", "0", "0"] and corner[4][1:4] == ["0", "0", "1"]
    from planner_cases import WEIGHTED
    exact = run(["plan 26 2 8 %d %s" % (m, fmt(WEIGHTED)) for m in (13, 12)])    # room for exactly the 13 steps, and one short
    assert exact[0][1:4] == ["0", "13", "0"] and exact[1][1:3] == ["-2", "13"]
    tiers = synthetic_tiers(2024, 4, rps_scale=400.0)
    lines.append("plan 128 4 8 2 %s" % " ".join(
        "%r %s %s" % (float(t[0]), " ".join(repr(float(x)) for x in t[1]), " ".join(repr(float(x)) for x in t[2])) for t in tiers))
    out = run(lines)
    for o, (allocs, left) in zip(out[:-1], want):
        assert o[:4] == ["plan", "0", str(len(allocs)), str(left)]
        vals = o[4:]
        for i, a in enumerate(allocs):
            f = vals[7 * i:7 * i + 7]
            assert [int(x) for x in f[:6]] == [a.tier, a.tp_prefill, a.tp_decode, a.P, a.D, a.gpus]
            assert float(f[6]) == a.served
    assert out[-1][1] == "-2" and int(out[-1][2]) > 2                # more steps than max_out: NTS_ERANGE, first two valid
    assert len(out[-1]) == 4 + 2 * 7
