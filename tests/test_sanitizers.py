"""The host code of the library (csrc/pd_host.cpp) and the C layer oracle built with
-fsanitize=address,undefined and run on the allocation model, the queue replays and a small layer
(dense and mixture of experts; exact and 8-bit cache; 8-bit activations; capacity errors): the run
must be clean, and its results must be the bytes an unsanitised build of the same driver writes
and the values the ordinary libraries return through their Python front ends."""
import os
import struct
import subprocess

import numpy as np
import pytest

import pd_inputs as I
from oracle import allocator as A
from oracle import layer as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = [os.path.join(ROOT, "tests", "sanitizer_driver.cpp"),
       os.path.join(ROOT, "paper_2603_04716_amd", "csrc", "pd_host.cpp")]
ORACLE_C = os.path.join(ROOT, "oracle", "layer_oracle.c")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]


def build(tmp, name, extra):
    common = ["-O1", "-g", "-ffp-contract=off", "-fopenmp", "-Wall", *extra]
    obj = os.path.join(tmp, name + "_oracle.o")
    subprocess.run(["gcc", "-std=c11", *common, "-c", ORACLE_C, "-o", obj], check=True)
    exe = os.path.join(tmp, name)
    subprocess.run(["g++", "-std=c++17", *common, "-I", os.path.join(ROOT, "include"), *SRC, obj, "-o", exe, "-lm"],
                   check=True)
    return exe


def write_case(path, cfg, w, x, xdec, cu, max_len, arrival, service):
    E = cfg.get("n_experts", 0)
    hdr = np.zeros(16, np.int32)
    hdr[:12] = [cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["d_ff"], E,
                cfg.get("top_k", 0), x.shape[0], len(cu) - 1, xdec.shape[0], max_len, len(arrival)]
    with open(path, "wb") as f:
        f.write(hdr.tobytes())
        for n in ("g_attn", "w_q", "w_k", "w_v", "w_o", "g_ffn", "w_gate", "w_up", "w_down"):
            f.write(np.ascontiguousarray(w[n], np.float32).tobytes())
        if E:
            f.write(np.ascontiguousarray(w["w_router"], np.float32).tobytes())
        f.write(np.ascontiguousarray(x, np.float32).tobytes())
        f.write(np.ascontiguousarray(xdec, np.float32).tobytes())
        f.write(np.ascontiguousarray(cu, np.int32).tobytes())
        f.write(np.ascontiguousarray(arrival, np.float64).tobytes())
        f.write(np.ascontiguousarray(service, np.float64).tobytes())


@pytest.fixture(scope="module")
def drivers(tmp_path_factory):
    tmp = str(tmp_path_factory.mktemp("san"))
    return build(tmp, "driver_san", SAN), build(tmp, "driver_plain", []), tmp


@pytest.mark.parametrize("moe", [False, True])
def test_host_code_and_oracle_are_clean_under_asan_and_ubsan(drivers, moe):
    san, plain, tmp = drivers
    cfg = I.small_config(d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ff=48,
                         n_experts=4 if moe else 0, top_k=2 if moe else 0)
    w = I.layer_weights(cfg, std=0.1, with_router=moe)
    cu = np.array([0, 9, 9, 10, 23], np.int32)            # ragged, one empty, one single-token sequence
    T, B, max_len = 23, 3, 28                             # slot of the 13-token sequence: 13 + 3 + 13 > 28
    x = I.hidden(T, 32, seed=1)
    xdec = I.hidden(B, 32, seed=2)
    rng = np.random.default_rng(5)
    arrival = np.cumsum(rng.exponential(0.07, 300))
    service = rng.exponential(0.05, 300)
    case, out_s, out_p = (os.path.join(tmp, f"{n}_{int(moe)}") for n in ("case", "out_san", "out_plain"))
    write_case(case, cfg, w, x, xdec, cu, max_len, arrival, service)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    r = subprocess.run([san, case, out_s], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stderr[-3000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr and "LeakSanitizer" not in r.stderr, \
        r.stderr[-3000:]
    subprocess.run([plain, case, out_p], check=True, timeout=300)
    blob = open(out_s, "rb").read()
    assert blob == open(out_p, "rb").read()
    # the worked example through the sanitised allocator: 3 prefill and 4 decode instances, and the
    # same doubles as the Python oracle
    st, n_p, n_d, tp_eff, ratio = struct.unpack_from("<iiidd", blob, 0)
    ref = A.allocate(5e6 / 60.0, 6144.0, 512.0, 2.0, 0.020, 28300.0, [8, 34, 64], [0.012, 0.020, 0.031], 0.1)
    assert (st, n_p, n_d) == (0, 3, 4)
    assert tp_eff == ref["tp_prefill_eff"] and ratio == ref["ratio_pd"]
    off = struct.calcsize("<iiidd")
    assert struct.unpack_from("<iiii", blob, off) == (7, 8, 1, 1)      # TTFT / TPOT infeasible, two invalid calls
    # the first prefill output of the sanitised oracle equals the ordinary oracle library's
    ol = O.Layer(cfg, w)
    oc = O.KVCache(ol, 4, max_len)
    want = O.prefill(ol, x, cu, cache=oc, slots=[3, 2, 1, 0])
    key = want.astype(np.float32).tobytes()
    assert key in blob
