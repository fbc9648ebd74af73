"""The C ABI used from plain C: tests/c_abi_client.c (C99, gcc, only include/jot.h and the HIP
runtime API) decodes a small problem from files; its results are compared with the CPU oracle."""
import os
import subprocess
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from gen.bf16 import bf16_bits_to_f32, f32_to_bf16_bits  # noqa: E402
from harness import too_close  # noqa: E402
from oracle import jot_oracle as O  # noqa: E402

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def build_client(tmp_path) -> str:
    import paper_2602_11133_amd as J
    exe = str(tmp_path / "c_abi_client")
    libdir = os.path.dirname(J.library_path())
    subprocess.check_call([
        "gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-O1", "-I", os.path.join(ROOT, "include"),
        "-I", "/opt/rocm/include", "-o", exe, os.path.join(ROOT, "tests", "c_abi_client.c"),
        "-L", libdir, "-ljot", "-L", "/opt/rocm/lib", "-lamdhip64",
        "-Wl,-rpath,/opt/rocm/lib", "-Wl,-rpath," + libdir])
    return exe


@pytest.mark.parametrize("dtype,block", [(O.F32, 0), (O.BF16, 8)])
def test_plain_c_client_matches_the_oracle(tmp_path, dtype, block):
    if not torch.cuda.is_available():
        pytest.fail("this test needs the MI355X; there is no CPU fallback")
    print(f"[c client] dtype={dtype} block={block}", flush=True)
    sys.stdout.flush()
    exe = build_client(tmp_path)
    rng = np.random.default_rng(90 + dtype)
    B, L, V, gs, steps = 2, 40, 3001, 8, 4
    p = O.OracleParams(B=B, L=L, V=V, dtype=dtype, conf_mode=O.CONF_RATIO,
                       tau_max=float(np.float32(30.0)), tau_min=1.0, gamma=0.5, D=8,
                       eps=float(np.float32(1e-12)), gen_start=gs, block_size=block)
    masked = np.zeros((B, L), bool)
    masked[:, gs:] = True
    tokens = rng.integers(0, V, (B, L)).astype(np.int32)
    st = O.OracleState.init(p, tokens, masked)
    tokens.tofile(tmp_path / "tokens.i32")
    masked.astype(np.uint8).tofile(tmp_path / "masked.u8")
    target = rng.integers(0, V, (B, L))
    counts = []
    for n in range(1, steps + 1):
        lg = (rng.standard_normal((B, L, V)) * 2).astype(np.float32)
        np.put_along_axis(lg, target[..., None], (rng.uniform(4, 16, (B, L, 1)) * n / steps).astype(np.float32) + 5, -1)
        if dtype == O.BF16:
            lg = bf16_bits_to_f32(f32_to_bf16_bits(lg)).reshape(lg.shape)
        flat = lg.reshape(B * L, V)
        for _ in range(50):                                   # keep every decision well posed (inputs only)
            act = st.active_list()
            rows = flat[act] if dtype == O.F32 else f32_to_bf16_bits(flat[act])
            bad = too_close(st.evaluate(np.ascontiguousarray(rows)), L)
            if bad.size == 0:
                break
            for k in bad:
                flat[act[k], target.reshape(-1)[act[k]]] += 2.0
        act = st.active_list()
        rows = flat[act] if dtype == O.F32 else f32_to_bf16_bits(flat[act])
        st.step(np.ascontiguousarray(rows))
        counts.append(st.active_count())
        (lg if dtype == O.F32 else f32_to_bf16_bits(lg)).tofile(tmp_path / f"logits_{n}.bin")
    args = [exe, str(tmp_path), B, L, V, dtype, O.CONF_RATIO, 30.0, 1.0, 0.5, 8, gs, block, steps]
    out = subprocess.run([str(a) for a in args], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    got_tokens = np.fromfile(tmp_path / "out_tokens.i32", np.int32).reshape(B, L)
    got_masked = np.fromfile(tmp_path / "out_masked.u8", np.uint8).reshape(B, L).astype(bool)
    got_log = np.fromfile(tmp_path / "out_log.i32", np.int32).reshape(-1, 3)
    got_counts = np.fromfile(tmp_path / "out_counts.i64", np.int64)
    np.testing.assert_array_equal(got_tokens, st.tokens)
    np.testing.assert_array_equal(got_masked, st.masked)
    np.testing.assert_array_equal(got_log, np.array(st.commit_log, np.int32).reshape(-1, 3))
    np.testing.assert_array_equal(got_counts, np.array(counts[: got_counts.size], np.int64))
    assert len(st.commit_log) > 0
