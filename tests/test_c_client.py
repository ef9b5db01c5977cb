"""The boundary from C: tests/c_abi_client.c (plain C99, include/samp.h + the HIP runtime's C API) is compiled with
gcc against libsamp.so.  Without a GPU only the build is checked (the header must be valid C); on a GPU the client
runs a small mixed-precision encoder from a file of inputs and its output must equal the oracle's."""
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "c_abi_client.c")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build_client(tmp_path):
    import paper_2209_09130_amd as P
    from paper_2209_09130_amd import build as B
    if not os.path.exists(P.lib_path()):
        B.build(force=True)
    pkg = os.path.dirname(P.lib_path())
    exe = str(tmp_path / "c_abi_client")
    cmd = ["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-D__HIP_PLATFORM_AMD__", "-isystem", f"{ROCM}/include",
           f"-I{ROOT}/include", SRC, "-o", exe, f"-L{pkg}", "-lsamp", f"-L{ROCM}/lib", "-lamdhip64",
           f"-Wl,-rpath,{pkg}", f"-Wl,-rpath,{ROCM}/lib"]
    subprocess.run(cmd, check=True)
    return exe


def test_header_is_valid_c99_and_a_c_client_links(tmp_path):
    exe = build_client(tmp_path)
    assert os.path.exists(exe)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 1 and "usage" in r.stderr


@pytest.mark.gpu
@pytest.mark.parametrize("varlen", [False, True])
def test_c_client_runs_the_encoder_and_matches_the_oracle(tmp_path, varlen):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import oracle
    import samp_workloads as W
    w = W.Workload("c-client", 3, 128, 2, 256, 4, 40, (W.FULL_INT8, W.FULL_INT8 | W.P_UNSIGNED, W.FULL_INT8), varlen=varlen,
                   min_len=1, plain_params=False, calib_batch=4, calib_seq=40)
    wts = W.make_weights(w)
    hid, lens, mask = W.make_hidden(w)
    cfg = (w.layers, w.hidden, w.heads, w.ffn, w.ln_eps)
    sc = oracle.calibrate(*cfg, wts, W.make_calibration_batch(w))
    want = oracle.Encoder(*cfg, w.modes, wts, sc).forward(hid, lens)
    inp, outp = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(inp, "wb") as f:
        f.write(np.array([w.layers, w.hidden, w.heads, w.ffn, w.batch, w.seq, int(varlen)], np.int32).tobytes())
        f.write(np.float32(w.ln_eps).tobytes())
        f.write(np.array(w.modes, np.uint8).tobytes())
        for lw in wts:
            for k in ("w_qkv", "w_o", "w_ffn1", "w_ffn2"):
                f.write(np.ascontiguousarray(lw[k], np.float16).tobytes())
            for k in ("b_qkv", "b_o", "b_ffn1", "b_ffn2", "ln1_g", "ln1_b", "ln2_g", "ln2_b"):
                f.write(np.ascontiguousarray(lw[k], np.float32).tobytes())
        f.write(np.ascontiguousarray(sc, np.float32).tobytes())
        f.write(np.ascontiguousarray(hid, np.float16).tobytes())
        if varlen:
            f.write(np.ascontiguousarray(mask, np.int32).tobytes())
    exe = build_client(tmp_path)
    r = subprocess.run([exe, str(inp), str(outp)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    got = np.fromfile(outp, np.float16).reshape(hid.shape)
    assert np.array_equal(got, want)                   # Fully-Quant: bit-identical
