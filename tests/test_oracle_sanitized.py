"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host only): oracle/sanitize_driver.c runs
every oracle function on small deterministic inputs in exactly-sized heap buffers; any out-of-bounds access,
signed overflow or misaligned access aborts it.  Every line it prints is recomputed here through the ordinary
build of the oracle on the same inputs, so the two builds must agree bit for bit."""
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _floats(n, salt):
    i = np.arange(n, dtype=np.uint64)
    m = ((i + np.uint64(salt)) * np.uint64(2654435761)) & np.uint64(0xFFFFFFFF)
    return (((m >> np.uint64(8)) & np.uint64(0xFFFF)).astype(np.float32) / np.float32(32768.0) - np.float32(1.0)).astype(np.float32)


def _bytes(n, salt):
    i = np.arange(n, dtype=np.uint64)
    m = ((i + np.uint64(salt)) * np.uint64(2654435761)) & np.uint64(0xFFFFFFFF)
    return (m >> np.uint64(11)).astype(np.uint8).view(np.int8)


def _fnv(*arrays):
    h = 1469598103934665603
    for a in arrays:
        for b in np.ascontiguousarray(a).tobytes():
            h = ((h ^ b) * 1099511628211) & 0xFFFFFFFFFFFFFFFF
    return "%016x" % h


@pytest.fixture(scope="module")
def driver_lines(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_sanitized")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           os.path.join(ROOT, "oracle", "sanitize_driver.c"), os.path.join(ROOT, "oracle", "sw_oracle.c"), "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    p = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-4000:]
    lines = [line for line in p.stdout.splitlines() if " : " in line]
    assert p.stdout.strip().endswith("done") and len(lines) >= 40
    return lines


def test_sanitized_oracle_runs_clean_and_agrees_with_the_ordinary_build(driver_lines, oracle):
    for line in driver_lines:
        head, want = line.split(" : ")
        name, *params = head.split()
        p = [int(v) for v in params]
        if name in ("conv2d", "conv2d_s8", "requant_s8", "bias_relu", "conv2d_dilated"):
            N, Ci, Co, H, W, R, S, st, pad = p[:9]
            x, w = _floats(N * Ci * H * W, 1).reshape(N, Ci, H, W), _floats(Co * Ci * R * S, 2).reshape(Co, Ci, R, S)
            x8, w8 = _bytes(N * Ci * H * W, 3).reshape(N, Ci, H, W), _bytes(Co * Ci * R * S, 4).reshape(Co, Ci, R, S)
            if name == "conv2d":
                got = _fnv(*oracle.conv2d(x, w, st, pad))
            elif name == "conv2d_s8":
                got = _fnv(oracle.conv2d_s8(x8, w8, st, pad))
            elif name == "requant_s8":
                scale = (np.float32(0.001) * (np.float32(2.0) + _floats(Co, 5))).astype(np.float32)
                i = np.arange(Co, dtype=np.uint64)
                bias = ((((i + np.uint64(6)) * np.uint64(2654435761)) & np.uint64(0xFFFFFFFF)) >> np.uint64(18)).astype(np.int64) - 8192
                got = _fnv(oracle.conv2d_s8_requant(x8, w8, bias.astype(np.int32), scale, st, pad, bool(p[9])))
            elif name == "bias_relu":
                got = _fnv(*oracle.conv2d_bias_relu(x, w, _floats(Co, 7), st, pad, bool(p[9])))
            else:
                got = _fnv(*oracle.conv2d_dilated(x, w, st, pad, p[9]))
        elif name in ("depthwise", "pool2d"):
            N, C, H, W, R, S, st, pad = p[:8]
            x = _floats(N * C * H * W, 8).reshape(N, C, H, W)
            if name == "depthwise":
                got = _fnv(*oracle.conv2d_depthwise(x, _floats(C * R * S, 9).reshape(C, 1, R, S), st, pad))
            else:
                got = _fnv(*oracle.pool2d(x, R, S, st, pad, p[8]))
        elif name in ("conv1d", "pool1d"):
            rows, length, k, st = p[:4]
            x = _floats(rows * length, 10).reshape(rows, length)
            if name == "conv1d":
                got = _fnv(*oracle.conv1d(x, _floats(k, 11), st, p[4]))
            else:
                got = _fnv(*oracle.pool1d(x, k, st, p[4]))
        else:
            raise AssertionError(name)
        assert got == want, line
