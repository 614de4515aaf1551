"""AddressSanitizer + UndefinedBehaviorSanitizer over the host code of both sides: the GPU library's planner (compiled
host-only, no device code, no GPU) and the CPU checker, each driven by a small program of its own over the same list of
operator descriptions: the workloads of the other tests, the benchmark shapes, and seeded random primitive graphs,
valid and invalid."""
import glob
import os
import random
import shutil
import subprocess

import pytest

from syno_inputs import BF16, F32, Builder, workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "sanitize")
OUT = os.path.join(SRC, "_build")
CSRC = os.path.join(ROOT, "paper_2410_23745_amd", "csrc")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def wire_line(d):
    import oracle
    w = oracle.wire(d).tolist()
    return " ".join(str(v) for v in [len(w)] + w + [int(d.in_dtype), int(d.out_dtype)])


def random_graph(rng):
    """A random primitive graph: mostly valid, sometimes with a dangling or reused coordinate or a bad factor."""
    n_out = rng.randint(1, 4)
    b = Builder([(f"o{i}", rng.choice([1, 2, 3, 4, 6, 8, 12])) for i in range(n_out)])
    live = list(range(n_out))
    size = {i: s for i, (_, s) in enumerate(b.desc.out_dims)}
    wcoords = []
    for _ in range(rng.randint(0, 7)):
        kind = rng.choice(["reduce", "share", "split", "merge", "shift", "unfold", "stride", "expand"])
        if kind == "reduce":
            n = rng.choice([1, 2, 3, 5]); c = b.reduce(n); size[c] = n; live.append(c)
        elif not live:
            continue
        elif kind == "share":
            c = live.pop(rng.randrange(len(live))); x, w = b.share(c); size[x] = size[w] = size[c]; live.append(x); wcoords.append(w)
        elif kind == "split" and len(live) >= 2:
            i = live.pop(rng.randrange(len(live))); j = live.pop(rng.randrange(len(live)))
            v = b.split(i, j); size[v] = size[i] * size[j]; live.append(v)
        elif kind == "merge":
            c = live.pop(rng.randrange(len(live)))
            divs = [k for k in range(1, size[c] + 1) if size[c] % k == 0]
            B = rng.choice(divs) if rng.random() < 0.9 else size[c] + 1
            q, r = b.merge(c, B); size[q], size[r] = max(1, size[c] // B), B; live += [q, r]
        elif kind == "shift":
            c = live.pop(rng.randrange(len(live)))
            by = rng.choice(live) if live and rng.random() < 0.3 else -1
            v = b.shift(c, rng.randint(-5, 5), by=by, coef=rng.randint(-2, 2) if by >= 0 else 0); size[v] = size[c]; live.append(v)
        elif kind == "unfold" and len(live) >= 2:
            i = live.pop(rng.randrange(len(live))); j = live.pop(rng.randrange(len(live)))
            v = b.unfold(i, j); size[v] = size[i]; live.append(v)
        elif kind == "stride":
            c = live.pop(rng.randrange(len(live))); S = rng.choice([1, 2, 3]); v = b.stride(c, S); size[v] = S * size[c]; live.append(v)
        elif kind == "expand" and len(live) >= 2:
            b.expand(live.pop(rng.randrange(len(live))))
    rng.shuffle(live)
    rng.shuffle(wcoords)
    if rng.random() < 0.1 and live:
        live.append(live[0])              # a coordinate used twice
    if rng.random() < 0.1 and live:
        live.pop()                        # a coordinate nobody consumes
    k = rng.randint(0, len(live))
    wcoords += live[k:]
    return b.finish(live[:k], wcoords, rng.choice([F32, BF16]), rng.choice([F32, BF16]))


def descriptors():
    from test_abi import pixel_unshuffle_conv
    ds = [wl.conv2d(2, 3, 4, 5, 6), wl.conv2d(1, 2, 2, 4, 5, 4, 2), wl.conv2d(3, 24, 40, 13, 19), wl.conv2d(2, 8, 16, 9, 9, 5, 5),
          wl.conv2d(3, 40, 24, 13, 19, 3, 3, BF16, F32), wl.conv2d(2, 36, 20, 11, 16, 3, 3, BF16, BF16, (2, 3, 1, 0)),
          wl.conv2d(2, 16, 32, 7, 7, 1, 1), wl.conv2d(5, 16, 16, 5, 4, 3, 3, BF16, F32), wl.conv2d(1, 8, 8, 6, 60),
          wl.grouped_shift_unfold(2, 8, 8, 5, 4, 4, 3), wl.grouped_shift_unfold(3), wl.grouped_shift_unfold(2, 96, 96, 9, 11, 3, 3, BF16, F32, (2, 0, 3, 1)),
          wl.strided_depthwise(2, 3, 3, 4), wl.strided_depthwise(3, 20, 15, 15), wl.strided_depthwise(2, 6, 12, 12, 1),
          wl.matmul(3, 4, 5), wl.matmul(37, 29, 45), wl.matmul(64, 640, 200, BF16, F32), wl.matmul(9, 3, 7),
          wl.operator1_stage1(3, 16, 16, 5, 12, 4, 2), wl.operator1_stage1(2, 12, 24, 4, 7, 3, 2, 3, BF16, BF16),
          wl.operator1_stage2(2, 16, 9, 10, 1), wl.window_of_sums_1d(120, 3, 2), wl.window_of_sums_1d(90, 5, 3, "k"),
          wl.window_of_sums_1d(64, 3, 4, "s"), wl.pooled_conv2d(3, 24, 40, 13, 10, 2, 3), wl.shifted_scale(3, 5, 7, 12),
          wl.pixel_unshuffle(2, 3, 5, 8, 2), wl.pixel_unshuffle(1, 2, 4, 5, 3), pixel_unshuffle_conv(),
          # strided windows (gradients planned on the phase planes), windows over flattened axes, views with gaps
          wl.conv2d(3, 24, 40, 7, 9, 3, stride=2), wl.conv2d(5, 40, 48, 4, 6, 1, 1, BF16, F32, stride=2),
          wl.conv2d(2, 16, 24, 5, 9, 3, stride=3), wl.flat_window(3, 24, 40, 6, 10), wl.flat_window(2, 80, 40, 7, 7, 5, BF16, F32),
          wl.shifted_scale(4, 8, 16, 16)]
    # the benchmark shapes (planned only: the checker's driver skips what is too large to evaluate)
    for C, H in wl.RESNET18_STAGES:
        ds += [wl.conv2d(32, C, C, H, H), wl.conv2d(32, C, C, H, H, 3, 3, BF16, F32)]
    ds += [wl.grouped_shift_unfold(32), wl.grouped_shift_unfold(128), wl.strided_depthwise(64, 128, 28, 28),
           wl.matmul(8192, 2304, 768), wl.matmul(8192, 2304, 768, BF16, F32), wl.pixel_unshuffle(64, 128, 28, 28, 2),
           wl.conv2d(32, 64, 128, 28, 28, 3, stride=2), wl.conv2d(32, 64, 128, 28, 28, 1, 1, BF16, F32, stride=2)]
    ds += wl.make_operator1(32, 64, 56).descs
    rng = random.Random(20241127)
    ds += [random_graph(rng) for _ in range(300)]
    return ds


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd[:4])} ...\n{r.stdout[-2000:]}\n{r.stderr[-4000:]}"
    return r


@pytest.fixture(scope="module")
def listing():
    os.makedirs(OUT, exist_ok=True)
    path = os.path.join(OUT, "descriptors.txt")
    with open(path, "w") as f:
        f.write("\n".join(wire_line(d) for d in descriptors()) + "\n")
    return path


def test_checker_under_address_and_undefined_behaviour_sanitizers(listing):
    exe = os.path.join(OUT, "oracle_driver")
    run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", *SAN, "-o", exe, os.path.join(SRC, "oracle_driver.c"),
         os.path.join(ROOT, "oracle", "syno_oracle.c")])
    r = run([exe, listing], env=dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1"))
    assert "evaluated" in r.stdout and "runtime error" not in r.stderr, r.stderr[-2000:]


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not installed")
def test_planner_under_address_and_undefined_behaviour_sanitizers(listing):
    """Host code of every library source (planner, C ABI, the kernel families' host logic), compiled without device
    code; the device images the host objects refer to are replaced by empty ones, which is fine as long as nothing
    is launched."""
    from paper_2410_23745_amd.build import SOURCES
    flags = ["-x", "hip", "--cuda-host-only", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC",
             "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    for s in SAN:
        flags += ["-Xarch_host", s]
    procs = []
    objs = []
    for src in SOURCES + ["host_driver.cpp"]:
        path = os.path.join(SRC if src == "host_driver.cpp" else CSRC, src)
        obj = os.path.join(OUT, src + ".o")
        objs.append(obj)
        procs.append((src, subprocess.Popen(["hipcc", "-c", path, "-o", obj] + flags, stdout=subprocess.PIPE,
                                            stderr=subprocess.PIPE, text=True)))
    for src, p in procs:
        _, err = p.communicate()
        assert p.returncode == 0, f"{src}:\n{err[-3000:]}"
    # empty device images under the names the host objects expect
    syms = set()
    for line in run(["nm", "-u"] + objs).stdout.split():
        if line.startswith("__hip_fatbin_"):
            syms.add(line)
    stub = os.path.join(OUT, "fatbin_stub.cpp")
    with open(stub, "w") as f:
        for s in sorted(syms):
            f.write(f'extern "C" __attribute__((section(".hip_fatbin"), aligned(4096))) const unsigned char {s}[4096] = {{0}};\n')
    run(["g++", "-c", stub, "-o", stub + ".o"])
    exe = os.path.join(OUT, "host_driver")
    run(["hipcc", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", exe] + objs + [stub + ".o"])
    r = run([exe, listing], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
    assert "planned" in r.stdout and "runtime error" not in r.stderr, r.stderr[-2000:]
    print(r.stdout.strip())
