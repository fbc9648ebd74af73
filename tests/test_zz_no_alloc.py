"""The allocation-free entry point jot_step_static against jot_init_state + jot_step: same
kernels, working memory in the library's fixed array instead of a caller's workspace.  Two calls
in a row, the second on a smaller problem (the array keeps the first call's contents), then the
first again."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def make_case(seed, B, L, V, dtype, block_size, gen_start):
    rng = np.random.default_rng(seed)
    masked = np.zeros((B, L), bool)
    masked[:, gen_start:] = rng.random((B, L - gen_start)) < 0.8
    tokens = rng.integers(0, V, (B, L)).astype(np.int32)
    logits = rng.standard_normal((B, L, V)).astype(np.float32) * 2.0
    target = rng.integers(0, V, (B, L))
    boost = rng.uniform(0.0, 14.0, (B, L)).astype(np.float32)
    np.put_along_axis(logits, target[..., None], boost[..., None], -1)
    return dict(B=B, L=L, V=V, dtype=dtype, block_size=block_size, gen_start=gen_start, tokens=tokens,
                masked=masked, logits=logits)


def run_both(case):
    import gpu_harness
    import paper_2602_11133_amd as J
    c = case
    p = J.JotParams(B=c["B"], L=c["L"], V=c["V"], dtype=c["dtype"], conf_mode=J.JOT_CONF_RATIO, tau_max=90.0,
                    tau_min=1.0, gamma=0.5, D=8, eps=1e-12, gen_start=c["gen_start"], block_size=c["block_size"])
    tdt = torch.float32 if c["dtype"] == J.JOT_F32 else torch.bfloat16
    dev = torch.from_numpy(c["logits"]).cuda().to(tdt).contiguous()
    sb, sl = c["L"] * c["V"], c["V"]
    stream = torch.cuda.current_stream().cuda_stream
    # the existing entry points
    g = gpu_harness.GpuJot(p, c["tokens"], c["masked"])
    g.step(dev, stride_b=sb, stride_l=sl)
    want = (g.tokens().copy(), g.masked().copy(), g.active_list().copy(), g.active_count())
    g.close()
    # the allocation-free one: canvas in and out through the caller's arrays
    n = c["B"] * c["L"]
    tok = torch.from_numpy(c["tokens"]).cuda()
    msk = torch.from_numpy(c["masked"].astype(np.uint8)).cuda()
    act = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((1,), -7, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    J.jot_step_static(p, dev.data_ptr(), sb, sl, tok.data_ptr(), msk.data_ptr(), act.data_ptr(), cnt.data_ptr(), stream)
    torch.cuda.synchronize()
    n_act = int(cnt.item())
    got = (tok.cpu().numpy(), msk.cpu().numpy().astype(bool), act.cpu().numpy()[:n_act], n_act)
    assert (act.cpu().numpy()[n_act:] == -7).all()          # nothing written beyond the list
    return want, got


def test_static_entry_point_matches_jot_step_on_two_calls_in_a_row():
    if not torch.cuda.is_available():
        pytest.fail("needs the MI355X")
    import paper_2602_11133_amd as J
    big = make_case(1, B=6, L=700, V=5004, dtype=J.JOT_F32, block_size=0, gen_start=60)
    small = make_case(2, B=1, L=70, V=1000, dtype=J.JOT_BF16, block_size=16, gen_start=6)
    for name, case in (("big", big), ("small", small), ("big again", big)):
        print(f"[static] {name}: B={case['B']} L={case['L']} V={case['V']} dtype={case['dtype']}", flush=True)
        want, got = run_both(case)
        np.testing.assert_array_equal(got[0], want[0])       # tokens
        np.testing.assert_array_equal(got[1], want[1])       # mask
        np.testing.assert_array_equal(got[2], want[2])       # next examined list
        assert got[3] == want[3]
        assert (want[1] != case["masked"]).any() and want[3] > 0     # the step did finalize something, not all


def test_static_entry_point_replayed_from_a_captured_graph():
    """The callers this entry point is for: one call is captured into a HIP graph (after an eager
    first call, which looks up the scratch address) and replayed; the canvas is carried from replay
    to replay through the caller's arrays.  Between replays the program does eager work, and every
    replay is compared with jot_init_state + jot_step on the same canvas and logits."""
    if not torch.cuda.is_available():
        pytest.fail("needs the MI355X")
    import gpu_harness
    import paper_2602_11133_amd as J
    c = make_case(3, B=2, L=300, V=4096, dtype=J.JOT_F32, block_size=0, gen_start=20)
    p = J.JotParams(B=c["B"], L=c["L"], V=c["V"], dtype=c["dtype"], conf_mode=J.JOT_CONF_RATIO, tau_max=90.0,
                    tau_min=1.0, gamma=0.5, D=8, eps=1e-12, gen_start=c["gen_start"], block_size=0)
    n = c["B"] * c["L"]
    sb, sl = c["L"] * c["V"], c["V"]
    rng = np.random.default_rng(4)
    logits = torch.from_numpy(c["logits"]).cuda()
    tok = torch.from_numpy(c["tokens"]).cuda()
    msk = torch.from_numpy(c["masked"].astype(np.uint8)).cuda()
    act = torch.zeros(n, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")

    def expected(tokens, masked, lg):
        g = gpu_harness.GpuJot(p, tokens, masked)
        g.step(lg, stride_b=sb, stride_l=sl)
        out = (g.tokens().copy(), g.masked().copy(), g.active_list().copy())
        g.close()
        return out

    def check(want):
        torch.cuda.synchronize()
        k = int(cnt.item())
        np.testing.assert_array_equal(tok.cpu().numpy(), want[0])
        np.testing.assert_array_equal(msk.cpu().numpy().astype(bool), want[1])
        np.testing.assert_array_equal(act.cpu().numpy()[:k], want[2])
        return want[0], want[1]

    # eager first call
    want = expected(c["tokens"], c["masked"], logits)
    J.jot_step_static(p, logits.data_ptr(), sb, sl, tok.data_ptr(), msk.data_ptr(), act.data_ptr(), cnt.data_ptr(),
                      torch.cuda.current_stream().cuda_stream)
    tokens, masked = check(want)
    # capture one call
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        J.jot_step_static(p, logits.data_ptr(), sb, sl, tok.data_ptr(), msk.data_ptr(), act.data_ptr(),
                          cnt.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    tok.copy_(torch.from_numpy(tokens)); msk.copy_(torch.from_numpy(masked.astype(np.uint8)))   # capture ran nothing
    for k in range(3):
        # eager work between replays: new logits for the next "denoising step", in place
        boost = torch.from_numpy((rng.uniform(0.0, 6.0, (c["B"], c["L"], 1))).astype(np.float32)).cuda()
        logits.add_(torch.where(logits > 8.0, boost, torch.zeros_like(boost)))
        torch.cuda.synchronize()
        want = expected(tokens, masked, logits)
        graph.replay()
        tokens, masked = check(want)
    assert not np.array_equal(masked, c["masked"])


def test_static_entry_point_rejects_what_does_not_fit():
    import paper_2602_11133_amd as J
    p = J.JotParams(B=64, L=1280, V=1000, dtype=J.JOT_F32, conf_mode=J.JOT_CONF_RATIO, tau_max=90.0, tau_min=1.0,
                    gamma=0.5, D=8, eps=1e-12, gen_start=0, block_size=0)
    assert J.jot_workspace_bytes(p) > J.JOT_STATIC_MAX_WORKSPACE
    with pytest.raises(J.JotError) as e:
        J.jot_step_static(p, 16, 1280 * 1000, 1000, 16, 16, 16, 16, 0)      # rejected before any pointer is used
    assert e.value.code == -10 and "scratch" in str(e.value)
