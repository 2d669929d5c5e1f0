"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer, on the CPU.

The host side of the library (aiq_host.cpp: validation, graph planning, workspace layout, launch sequencing)
is compiled with g++ against stand-ins for the HIP runtime and for the kernel launchers
(tests/host_sanitize/hip_stub.cpp: "device" memory is host memory, every launcher touches the extents its
kernel would read and write), the oracle (oracle/oracle.c) with gcc, both with -fsanitize=address,undefined,
and one driver runs every entry point over the model families and over seeded random graphs.  A sanitizer
report aborts the driver; a wrong status fails it.  Nothing here touches a GPU.
"""
import os
import struct
import subprocess

import numpy as np
import pytest

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "host_sanitize")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


def _random_graph(rng):
    G = synth.graphs
    ci, h = int(rng.choice([1, 3, 4])), int(rng.integers(6, 21))
    widths = [8, 12, 16, 24, 40, 64, 100]
    c = int(rng.choice(widths))
    nodes = [G._node(G.KIND_CONV, ci, c, 3, 1, h, -1, act=int(rng.integers(0, 3)), slot=0)]
    shapes = [(c, h)]
    for i in range(int(rng.integers(3, 7))):
        c_in, h_in = shapes[-1]
        kind = str(rng.choice(["c3", "c3", "c1", "dw", "c3s2", "dws2", "c1s2"]))
        stride = 2 if kind.endswith("s2") and h_in >= 4 else 1
        k = 1 if kind.startswith("c1") else 3
        h_out = (h_in + 2 * (k // 2) - k) // stride + 1
        if kind.startswith("dw"):
            nodes.append(G._node(G.KIND_DEPTHWISE, c_in, c_in, 3, stride, h_in, len(nodes) - 1, act=int(rng.integers(0, 3)),
                                 slot=len(nodes)))
            shapes.append((c_in, h_out))
            continue
        c_out = int(rng.choice(widths))
        cands = [j for j, (cj, hj) in enumerate(shapes) if hj == h_out]
        res = -1
        if cands and rng.random() < 0.5:
            res = int(rng.choice(cands))
            c_out = shapes[res][0]
        nodes.append(G._node(G.KIND_CONV, c_in, c_out, k, stride, h_in, len(nodes) - 1, residual=res,
                             act=int(rng.integers(0, 3)), slot=len(nodes)))
        shapes.append((c_out, h_out))
    c_last, h_last = shapes[-1]
    nodes.append(G._node(G.KIND_FC, c_last, int(rng.choice([2, 10, 37])), 1, 1, h_last, len(nodes) - 1, slot=len(nodes)))
    return nodes


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = tmp_path_factory.mktemp("host_sanitize")
    exe = str(out / "driver")
    inc = ["-I/opt/rocm/include", "-D__HIP_PLATFORM_AMD__"]
    objs = []
    for src, cc, extra in ((os.path.join(ROOT, "paper_2512_14090_amd", "csrc", "aiq_host.cpp"), "g++", ["-std=c++17"] + inc),
                           (os.path.join(HERE, "hip_stub.cpp"), "g++", ["-std=c++17"] + inc),
                           (os.path.join(HERE, "driver.cpp"), "g++", ["-std=c++17"]),
                           (os.path.join(ROOT, "oracle", "oracle.c"), "gcc",
                            ["-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math"])):
        obj = str(out / (os.path.basename(src) + ".o"))
        subprocess.run([cc] + SAN + extra + ["-Wall", "-c", src, "-o", obj], check=True)
        objs.append(obj)
    subprocess.run(["g++"] + SAN + objs + ["-fopenmp", "-lm", "-o", exe], check=True)
    return exe, out


def test_host_side_and_oracle_under_asan_ubsan(driver):
    exe, out = driver
    # (graph, images for the oracle pass: 0 = library only - the oracle's direct loops are slow under ASan)
    graphs = [(synth.resnet_cifar(1), 2), (synth.resnet_cifar(3), 0), (synth.mobilenetv2_32(), 0),
              (synth.plain_convnet20(), 0), (synth.heavy_early_resnet20(), 0)]
    rng = np.random.Generator(np.random.PCG64(2024))
    graphs += [(_random_graph(rng), 2) for _ in range(10)]
    path = str(out / "graphs.bin")
    with open(path, "wb") as f:
        f.write(struct.pack("<i", len(graphs)))
        for nodes, n_img in graphs:
            d = synth.desc_array(nodes)
            f.write(struct.pack("<ii", d.shape[0], n_img))
            f.write(d.astype("<i4").tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    r = subprocess.run([exe, path], capture_output=True, text=True, env=env, timeout=900)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "HOST SANITIZE OK" in r.stdout, tail
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, tail
