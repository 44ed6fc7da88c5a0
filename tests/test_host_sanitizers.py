"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the library's model-file loader (header
checks, re-layout of the weights into the device image) and the two C oracles, built into one small
program (tests/sanitize/driver.cpp) and run on good and broken inputs.  Any report aborts the program
(-fno-sanitize-recover), which fails the test; results must also equal those of the ordinary builds."""
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import anticipator as oa
from oracle import lookahead as ol
from paper_2504_03702_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2504_03702_amd", "csrc")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("sanitize") / "driver")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan"]
    objs = []
    for src in (os.path.join(ROOT, "oracle", "anticipator.c"), os.path.join(ROOT, "oracle", "lookahead.c")):
        obj = out + "_" + os.path.basename(src) + ".o"
        subprocess.check_call(["gcc", "-g", "-O1", "-std=c99", "-Wall", *san[:2], "-c", src, "-o", obj])
        objs.append(obj)
    subprocess.check_call(["g++", "-g", "-O1", "-std=c++17", "-Wall", *san, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                           os.path.join(ROOT, "tests", "sanitize", "driver.cpp"), os.path.join(CSRC, "model_file.cpp"),
                           *objs, "-o", out])
    return out


def run(driver, *args):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([driver, *args], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, f"{args}: exit {r.returncode}\n{r.stdout}\n{r.stderr}"
    return r.stdout


def test_model_loader_on_good_and_broken_files(driver, tmp_path):
    small_bf16 = wl.ModelConfig(layers=2, hidden=256, heads=4, ffn=512, vocab=300, max_pos=64, n_soft=3,
                                head_hidden=40, dtype=wl.DTYPE_BF16)
    tiny = wl.MODELS["tiny"]
    good = {}
    for name, cfg in (("tiny", tiny), ("bf16", small_bf16)):
        path = str(tmp_path / f"{name}.bin")
        wl.write_model(path, cfg, wl.make_weights(cfg, seed=0, ln_jitter=0.1, bias_std=0.05))
        good[name] = path
        out = run(driver, "model", path)
        assert out.splitlines()[0] == "rc 0" and f"layers {cfg.layers} " in out
        assert out == run(driver, "model", path)                      # the same image twice
    raw = open(good["bf16"], "rb").read()

    def variant(name, data):
        p = str(tmp_path / name)
        with open(p, "wb") as f:
            f.write(data)
        return run(driver, "model", p).splitlines()[0]

    assert variant("empty.bin", b"") == "rc -3"
    assert variant("short_header.bin", raw[:40]) == "rc -3"
    assert variant("bad_magic.bin", b"X" + raw[1:]) == "rc -3"
    assert variant("truncated.bin", raw[:-2]) == "rc -3"
    assert variant("one_more.bin", raw + b"\0\0") == "rc -3"
    hdr = list(struct.unpack_from("<10i", raw, 8))
    def with_header(i, v):
        h = list(hdr)
        h[i] = v
        return raw[:8] + struct.pack("<10i", *h) + raw[48:]
    assert variant("zero_layers.bin", with_header(0, 0)) == "rc -3"
    assert variant("huge_layers.bin", with_header(0, 2**31 - 1)) == "rc -3"
    assert variant("huge_vocab.bin", with_header(4, 2**31 - 1)) == "rc -3"
    assert variant("negative_soft.bin", with_header(6, -1)) == "rc -3"
    assert variant("heads_do_not_divide.bin", with_header(2, 3)) == "rc -3"
    assert variant("bad_dtype.bin", with_header(8, 7)) == "rc -3"
    # a consistent file the bf16 kernels are not built for: head size 32
    odd = wl.ModelConfig(layers=1, hidden=256, heads=8, ffn=256, vocab=50, max_pos=16, dtype=wl.DTYPE_BF16)
    p = str(tmp_path / "odd.bin")
    wl.write_model(p, odd, wl.make_weights(odd, seed=1))
    assert run(driver, "model", p).splitlines()[0] == "rc -6"


def pack(n, n_inst, length, flag, map0, ovf0, *cols):
    parts = [struct.pack("<q4i", n, n_inst, length, flag, 0), np.ascontiguousarray(map0, np.int32).tobytes(),
             np.ascontiguousarray(ovf0, np.int64).tobytes()]
    parts += [np.ascontiguousarray(c, np.int32).tobytes() for c in cols]
    return b"".join(parts)


def unpack(path, n_inst, length):
    raw = open(path, "rb").read()
    rc, bad = struct.unpack_from("<2q", raw, 0)
    m = np.frombuffer(raw, np.int32, n_inst * length, 16).reshape(n_inst, length)
    o = np.frombuffer(raw, np.int64, n_inst, 16 + 4 * n_inst * length)
    return rc, bad, m, o


def test_oracles_under_sanitizers_match_the_plain_builds(driver, tmp_path):
    rng = np.random.default_rng(0)
    # anticipator: with and without rates, faulty records of every kind, an arrival in the last bucket, a bucket
    # pushed over the int32 range
    for with_rate in (True, False):
        inp = wl.make_anticipator_inputs("medium" if with_rate else "tiny", seed=3, n=5000)
        pred, inst, arr = inp.pred_tokens.copy(), inp.instance_id.copy(), inp.arrival_bucket.copy()
        pred[[5, 77]] = [-1, 0]
        inst[[9, 400]] = [inp.n_inst, -4]
        arr[[11, 12, 13]] = [inp.horizon, -1, inp.horizon - 1]
        load0 = rng.integers(-9, 9, (inp.n_inst, inp.horizon)).astype(np.int32)
        load0[0, 0] = 2**31 - 1
        ovf0 = rng.integers(0, 50, inp.n_inst).astype(np.int64)
        src, dst = str(tmp_path / "a.in"), str(tmp_path / "a.out")
        rate = inp.rate if with_rate else np.zeros(0, np.int32)
        with open(src, "wb") as f:
            f.write(pack(len(pred), inp.n_inst, inp.horizon, int(with_rate), load0, ovf0, pred, inst, arr, rate))
        run(driver, "anticipate", src, dst)
        rc, bad, m, o = unpack(dst, inp.n_inst, inp.horizon)
        want_m, want_o, want_rc, want_bad = oa.anticipate(pred, inst, arr, inp.rate if with_rate else None, inp.n_inst,
                                                          inp.horizon, load=load0, overflow=ovf0)
        assert (rc, bad) == (want_rc, want_bad) and rc & 1
        assert np.array_equal(m, want_m) and np.array_equal(o, want_o)
    # look-ahead map: ramps that cross the end of the map, corrections, faulty records
    x = wl.make_lookahead_inputs("medium", seed=4)
    cols = [c.copy() for c in x.columns()]
    cols[0][3] = x.n_inst
    cols[1][4] = x.map_len
    cols[4][5] = 70000
    cols[5][6] = 0
    n = len(cols[0])
    src, dst = str(tmp_path / "l.in"), str(tmp_path / "l.out")
    with open(src, "wb") as f:
        f.write(pack(n, x.n_inst, x.map_len, 0, np.zeros((x.n_inst, x.map_len), np.int32), np.zeros(x.n_inst, np.int64), *cols))
    run(driver, "lookahead", src, dst)
    rc, bad, m, o = unpack(dst, x.n_inst, x.map_len)
    want_m, want_o, want_rc, want_bad = ol.lookahead_update(*cols, x.n_inst, x.map_len)
    assert (rc, bad) == (want_rc, want_bad) and bad == 3
    assert np.array_equal(m, want_m) and np.array_equal(o, want_o)
