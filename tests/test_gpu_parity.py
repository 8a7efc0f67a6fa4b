"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same seeded
inputs.  Bars: max-normalised error <= 1e-3 (fp32 storage) / 2e-2 (bf16 storage) per tensor."""
import numpy as np
import pytest
import torch

import paper_2411_19460_amd as pk
from oracle import ssd_ref
from paper_2411_19460_amd import synth
from parity_util import TOL, check, compare_all, dev_inputs, host, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


def small_inputs(seed, dtype, Bt, L, H, P, G, N, states=True):
    cfg = synth.SSDConfig("t", dtype, Bt, L, H, P, N, G, 1, L, index=50 + seed)
    return synth.make_layer_inputs(cfg, with_states=states)


def test_config0_fp32_all_tensors():
    cfg = synth.CONFIGS[0]
    d = synth.make_layer_inputs(cfg)
    rep = {}
    compare_all(d, cfg.dtype, cfg.chunk, cfg.segment, report=rep)
    print("config0 errors:", {k: f"{v:.2e}" for k, v in rep.items()})


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [
    # Bt, L,  H, P,  G, N,  Q,  segment  : ragged tiles (P, N, Q not multiples of 32), groups, batch
    (2, 192, 4, 24, 2, 40, 48, 96),
    (1, 256, 6, 16, 3, 16, 64, 64),
    (1, 130, 2, 8, 1, 8, 1, 13),       # chunk of one token
    (1, 96, 2, 33, 1, 65, 96, 96),     # one chunk, one segment
])
def test_generic_kernels_odd_shapes_with_states(dtype, shape):
    Bt, L, H, P, G, N, Q, seg = shape
    d = small_inputs(1, dtype, Bt, L, H, P, G, N)
    compare_all(d, dtype, Q, seg, flags=pk.SSD_FLAG_GENERIC_KERNELS)


def test_segmentation_does_not_change_results():
    # MA-GC's sequence axis is exact (Markov property): segment = 64 vs no checkpoints at all.
    d = small_inputs(2, "f32", 1, 512, 4, 16, 1, 16)
    dv = dev_inputs(d, "f32")
    y1, f1, _, g1 = run_gpu(dv, 64, 64)
    y2, f2, _, g2 = run_gpu(dv, 64, None)
    assert torch.equal(y1, y2) and torch.equal(f1, f2)
    for k in g1:
        a, b = host(g1[k]), host(g2[k])
        assert np.max(np.abs(a - b)) <= 1e-5 * max(1e-30, np.max(np.abs(b))), k
    for k in ("dx", "ddt", "dB", "dC", "dinit_state"):
        assert torch.equal(g1[k], g2[k]), k   # same kernels, same order: bitwise


def test_residual_and_accumulate_flags():
    d = small_inputs(3, "f32", 1, 128, 2, 16, 1, 16)
    compare_all(d, "f32", 32, 64, flags=pk.SSD_FLAG_RESIDUAL, residual=True)
    dv = dev_inputs(d, "f32")
    _, _, bnd = pk.ssd_fwd(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], 32, 64, dv["init_state"])
    g0 = pk.ssd_bwd(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], dv["dy"], 32, 64, dv["init_state"],
                    dv["dfinal_state"], bnd)
    dA = torch.full_like(g0["dA"], 3.0)
    dD = torch.full_like(g0["dD"], -2.0)
    pk.ssd_bwd(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], dv["dy"], 32, 64, dv["init_state"],
               dv["dfinal_state"], bnd, flags=pk.SSD_FLAG_ACCUM_PARAM, dA=dA, dD=dD)
    assert torch.allclose(dA, g0["dA"] + 3.0, rtol=1e-6, atol=1e-6)
    assert torch.allclose(dD, g0["dD"] - 2.0, rtol=1e-6, atol=1e-6)


def test_empty_sequence_passes_state_through():
    H, P, N = 2, 8, 8
    x = torch.empty((1, 0, H, P), device="cuda")
    dt = torch.empty((1, 0, H), device="cuda")
    Bm = torch.empty((1, 0, 1, N), device="cuda")
    A = -torch.ones(H, device="cuda")
    D = torch.ones(H, device="cuda")
    init = torch.randn((1, H, P, N), device="cuda")
    y, fin, _ = pk.ssd_fwd(x, dt, A, Bm, Bm, D, 64, None, init)
    assert y.numel() == 0 and torch.equal(fin, init)
    g = pk.ssd_bwd(x, dt, A, Bm, Bm, D, x, 64, None, init, init * 2)
    assert torch.equal(g["dinit_state"], init * 2) and float(g["dA"].abs().sum()) == 0.0


@pytest.mark.parametrize("shape", [
    # Bt, L,   H, G, Q,   segment      (P = 64, N = 128: the matrix-core path)
    (2, 512, 4, 2, 64, 256),
    (1, 768, 3, 1, 128, 384),
    (1, 1024, 4, 1, 256, 512),
    (2, 512, 2, 2, 256, 512),
])
def test_mfma_path_small_with_states(shape):
    Bt, L, H, G, Q, seg = shape
    d = small_inputs(4, "bf16", Bt, L, H, 64, G, 128)
    rep = {}
    dv, (y, fin, bnd, g) = compare_all(d, "bf16", Q, seg, report=rep)
    print("mfma errors:", {k: f"{v:.2e}" for k, v in rep.items()})
    # and against the shape-generic kernels on the device (same algorithm, fp32 FMA arithmetic)
    y2, fin2, bnd2, g2 = run_gpu(dv, Q, seg, flags=pk.SSD_FLAG_GENERIC_KERNELS)
    check("y vs generic", host(y), host(y2), 2e-2)
    for k in g:
        check(k + " vs generic", host(g[k]), host(g2[k]), 2e-2)


def test_mfma_residual_flag():
    d = small_inputs(5, "bf16", 1, 512, 2, 64, 1, 128)
    compare_all(d, "bf16", 256, 256, flags=pk.SSD_FLAG_RESIDUAL, residual=True)


def test_config1_bf16_generic_kernels():
    cfg = synth.CONFIGS[1]
    d = synth.make_layer_inputs(cfg)
    compare_all(d, cfg.dtype, cfg.chunk, cfg.segment, flags=pk.SSD_FLAG_GENERIC_KERNELS)


def test_config1_bf16_all_tensors():
    cfg = synth.CONFIGS[1]
    d = synth.make_layer_inputs(cfg)
    rep = {}
    compare_all(d, cfg.dtype, cfg.chunk, cfg.segment, report=rep)
    print("config1 errors:", {k: f"{v:.2e}" for k, v in rep.items()})


@pytest.mark.parametrize("path", ["mfma", "generic"])
def test_padding_tokens_and_extreme_decay(path):
    """dt = 0 tokens (padding: the state passes through, the token adds nothing) and dt of order 5 (the
    state is forgotten within a token or two; cum reaches -2e4 inside a chunk): every factor of the
    decay mask stays <= 1, so nothing may overflow or turn into NaN, and the results still match."""
    Bt, L, H, G, Q, seg = 1, 512, 4, 1, 256, 256
    d = small_inputs(9, "bf16", Bt, L, H, 64, G, 128)
    rng = np.random.default_rng(5)
    dt = d["dt"].copy()
    dt[:, 100:140] = 0.0                      # a run of padding tokens inside a chunk
    dt[:, 250:262] = 0.0                      # ... and across a chunk boundary
    dt[:, 300:330, 1] = 5.0                   # head 1: extreme decay for a while
    dt[:, :, 3] = np.where(rng.random((Bt, L)) < 0.3, 4.0, dt[:, :, 3])   # head 3: extreme decay at random tokens
    d["dt"] = synth.round_bf16(dt)
    flags = pk.SSD_FLAG_GENERIC_KERNELS if path == "generic" else 0
    rep = {}
    compare_all(d, "bf16", Q, seg, flags=flags, report=rep)
    print("padding/extreme-decay errors:", {k: f"{v:.2e}" for k, v in rep.items()})


def test_autograd_wrapper_matches_the_direct_calls_and_the_oracle():
    d = small_inputs(11, "bf16", 2, 512, 4, 64, 2, 128)
    dv = dev_inputs(d, "bf16")
    leaf = {k: dv[k].clone().requires_grad_(True) for k in ("x", "dt", "A", "B", "C", "D", "init_state")}
    y, fin = pk.ssd_scan(leaf["x"], leaf["dt"], leaf["A"], leaf["B"], leaf["C"], leaf["D"], 256, 256, leaf["init_state"])
    loss = (y.float() * dv["dy"].float()).sum() + (fin * dv["dfinal_state"]).sum()
    loss.backward()
    torch.cuda.synchronize()
    _, _, _, g = run_gpu(dv, 256, 256)
    for k, gk in (("x", "dx"), ("dt", "ddt"), ("A", "dA"), ("B", "dB"), ("C", "dC"), ("D", "dD"), ("init_state", "dinit_state")):
        assert torch.equal(leaf[k].grad, g[gk]), k
    _, go = run_oracle(d, 256)
    check("dx via autograd", host(leaf["x"].grad), go["dx"], TOL["bf16"])
    check("dA via autograd", host(leaf["A"].grad), go["dA"], TOL["bf16"])


@pytest.mark.parametrize("case", [
    # dtype, Bt, L,    H, P,  G, N,   Q,   segment, flags
    ("f32", 2, 200, 3, 16, 1, 16, 64, 128, 0),                                 # short last segment, short last chunk
    ("bf16", 2, 1000, 4, 64, 2, 128, 256, 512, 0),                             # matrix-core path, two segments in flight
    ("bf16", 1, 300, 2, 64, 1, 128, 256, None, 0),                             # one segment, shorter than two chunks
    ("bf16", 1, 2148, 2, 64, 1, 128, 128, 512, 0),                             # five segments on four lanes, tail of 100
    ("bf16", 1, 700, 2, 64, 1, 128, 128, 256, pk.SSD_FLAG_GENERIC_KERNELS),
])
def test_sequence_length_need_not_be_a_multiple_of_segment_or_chunk(case):
    dtype, Bt, L, H, P, G, N, Q, seg, flags = case
    d = small_inputs(13, dtype, Bt, L, H, P, G, N)
    dv = dev_inputs(d, dtype)
    y, fin, bnd, g = run_gpu(dv, Q, seg, flags)
    f, go = run_oracle(d, None)
    tol = TOL[dtype]
    check("y", host(y), f["y"], tol)
    check("final_state", host(fin), f["final_state"], tol)
    if seg is not None:
        nseg = -(-L // seg)
        assert bnd.shape[1] == nseg
        for k in range(1, nseg):   # the state entering segment k = the final state of the first k segments
            fk = ssd_ref.ssd_fwd(d["x"][:, :k * seg], d["dt"][:, :k * seg], d["A"], d["B"][:, :k * seg], d["C"][:, :k * seg],
                                 d["D"], d["init_state"])
            check(f"boundary_states[{k}]", host(bnd[:, k]), fk["final_state"], tol)
    for k in ("dx", "ddt", "dA", "dB", "dC", "dD", "dinit_state"):
        check(k, host(g[k]), go[k], tol)
    # prefill without checkpoints agrees
    y2, fin2, _ = pk.ssd_fwd(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], Q, seg, dv["init_state"], flags,
                             want_boundary=False)
    torch.cuda.synchronize()
    assert torch.equal(y, y2) and torch.equal(fin, fin2)


@pytest.mark.parametrize("case", [
    # dtype, Bt, L,   H, P,  G, N,   Q,   segment, flags
    ("f32", 2, 256, 3, 16, 1, 16, 64, 128, 0),
    ("bf16", 2, 1024, 4, 64, 2, 128, 256, 512, 0),
    ("bf16", 1, 1100, 2, 64, 1, 128, 128, 256, 0),                             # five segments in flight, short tail
    ("bf16", 1, 768, 2, 64, 1, 128, 256, 256, pk.SSD_FLAG_GENERIC_KERNELS),
])
def test_packed_sequences(case):
    """seq_reset marks the first token of every packed sequence: starts inside a chunk, on a chunk
    boundary, on a segment boundary, two in a row, and at token 0 (which discards init_state)."""
    dtype, Bt, L, H, P, G, N, Q, seg, flags = case
    d = small_inputs(17, dtype, Bt, L, H, P, G, N)
    reset = np.zeros((Bt, L), dtype=np.uint8)
    for t in (37, Q, Q + 1, seg, seg + Q // 2, L - 3):
        reset[0, t] = 1
    if Bt > 1:
        reset[1, 0] = 1
        reset[1, L // 2 + 5] = 1
    dv = dev_inputs(d, dtype)
    rdev = torch.from_numpy(reset).cuda()
    y, fin, bnd = pk.ssd_fwd(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], Q, seg, dv["init_state"], flags,
                             seq_reset=rdev)
    g = pk.ssd_bwd(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], dv["dy"], Q, seg, dv["init_state"],
                   dv["dfinal_state"], bnd, flags, seq_reset=rdev)
    torch.cuda.synchronize()
    f = ssd_ref.ssd_fwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["init_state"], reset=reset)
    go = ssd_ref.ssd_bwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["dy"], d["init_state"], d["dfinal_state"],
                         reset=reset)
    tol = TOL[dtype]
    rep = {}
    check("y", host(y), f["y"], tol, rep)
    check("final_state", host(fin), f["final_state"], tol, rep)
    for k in ("dx", "ddt", "dA", "dB", "dC", "dD", "dinit_state"):
        check(k, host(g[k]), go[k], tol, rep)
    print("packed errors:", {k: f"{v:.2e}" for k, v in rep.items()})
    # row 1 starts with a reset: its initial state must not matter at all
    if Bt > 1:
        assert float(g["dinit_state"][1].abs().max()) <= 1e-30
    # the recurrent step honours the flags too
    state = dv["init_state"].clone()
    yd = pk.ssd_decode(dv["x"][:, :70].contiguous(), dv["dt"][:, :70].contiguous(), dv["A"], dv["B"][:, :70].contiguous(),
                       dv["C"][:, :70].contiguous(), dv["D"], state, seq_reset=rdev[:, :70].contiguous())
    torch.cuda.synchronize()
    check("y (decode)", host(yd), f["y"][:, :70], tol)


def _oracle_bwd_from_checkpoints(d, segment, ckpt):
    """The backward sweep of Alg. 2 written out with the oracle: segments right to left, each restarted
    from the stored checkpoint `ckpt[:, k]` (segment 0 from the initial state), the state adjoint handed
    to the left."""
    L = d["x"].shape[1]
    nseg = L // segment
    dstate = d.get("dfinal_state")
    segs = [None] * nseg
    for k in reversed(range(nseg)):
        sl = slice(k * segment, (k + 1) * segment)
        init = d.get("init_state") if k == 0 else ckpt[:, k]
        segs[k] = ssd_ref.ssd_bwd(d["x"][:, sl], d["dt"][:, sl], d["A"], d["B"][:, sl], d["C"][:, sl], d["D"],
                                  d["dy"][:, sl], init, dstate)
        dstate = segs[k]["dinit_state"]
    out = {k: np.concatenate([g[k] for g in segs], axis=1) for k in ("dx", "ddt", "dB", "dC")}
    out.update({k: sum(g[k] for g in segs) for k in ("dA", "dD")})
    out["dinit_state"] = dstate
    return out


@pytest.mark.parametrize("case", [
    # dtype, Bt, L, H, P, G, N, Q, segment, flags
    ("f32", 2, 512, 3, 16, 1, 16, 64, 128, 0),                      # shape-generic kernels
    ("bf16", 1, 2048, 4, 64, 2, 128, 256, 512, 0),                  # matrix-core kernels
    ("bf16", 1, 1024, 2, 64, 1, 128, 128, 256, pk.SSD_FLAG_GENERIC_KERNELS),
])
def test_bf16_checkpoints(case):
    # App. C: the S-checkpoint may be kept in bf16 (half the bytes).  The forward pass does not change;
    # the backward pass restarts every segment but the first from the rounded state.
    dtype, Bt, L, H, P, G, N, Q, seg, fl = case
    d = small_inputs(17, dtype, Bt, L, H, P, G, N)
    dv = dev_inputs(d, dtype)
    y32, fin32, bnd32, g32 = run_gpu(dv, Q, seg, fl)
    y16, fin16, bnd16, g16 = run_gpu(dv, Q, seg, fl | pk.SSD_FLAG_BF16_CHECKPOINTS)
    assert bnd16.dtype == torch.bfloat16 and bnd16.shape == bnd32.shape
    assert torch.equal(y16, y32) and torch.equal(fin16, fin32)
    assert torch.equal(bnd16, bnd32.to(torch.bfloat16))          # one rounding of the same fp32 state
    f = ssd_ref.ssd_fwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d.get("init_state"), seg)
    check("boundary_states", host(bnd16), f["boundary_states"], max(TOL[dtype], 2.0 ** -8))
    ref = _oracle_bwd_from_checkpoints(d, seg, synth.round_bf16(f["boundary_states"]).astype(np.float64))
    plain = ssd_ref.ssd_bwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["dy"], d.get("init_state"), d.get("dfinal_state"))
    rep = {}
    for k in ("dx", "ddt", "dA", "dB", "dC", "dD", "dinit_state"):
        check(k, host(g16[k]), ref[k], TOL[dtype], rep)
    print("bf16 checkpoints, error against the segment-wise oracle:", {k: f"{v:.2e}" for k, v in rep.items()})
    print("distance of that oracle from the exact gradients:",
          {k: f"{np.max(np.abs(ref[k] - plain[k])) / np.max(np.abs(plain[k])):.2e}" for k in ("dx", "ddt", "dA", "dC", "dinit_state")})
    # the wrong dtype for the flags is refused before anything is launched
    with pytest.raises(TypeError):
        pk.ssd_bwd(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], dv["dy"], Q, seg, dv.get("init_state"),
                   dv.get("dfinal_state"), bnd32, fl | pk.SSD_FLAG_BF16_CHECKPOINTS)


def test_fp32_chunk_states_flag():
    """SSD_FLAG_FP32_CHUNK_STATES: the scans read their per-chunk inputs in fp32 (App. C keeps SSM states in fp32)
    instead of the default bf16 copies; same results within the same bar, every tensor, states entering and
    leaving the sequence included; and nothing but rounding separates the two variants."""
    d = small_inputs(21, "bf16", 2, 1536, 4, 64, 2, 128)
    rep = {}
    dv, (y, fin, bnd, g) = compare_all(d, "bf16", 256, 512, flags=pk.SSD_FLAG_FP32_CHUNK_STATES, report=rep)
    print("fp32 chunk states, errors:", {k: f"{v:.2e}" for k, v in rep.items()})
    y0, fin0, bnd0, g0 = run_gpu(dv, 256, 512)
    for a, b in ((y, y0), (fin, fin0), (g["dx"], g0["dx"]), (g["dB"], g0["dB"]), (g["dinit_state"], g0["dinit_state"])):
        assert float((a.float() - b.float()).abs().max()) <= 2.0 ** -6 * float(b.float().abs().max())


def test_forward_and_backward_can_be_captured_in_a_graph():
    """The calls enqueue only kernels and event record/wait pairs (no memset, no allocation, no host
    synchronisation), on the caller's stream and on the library's own streams forked from it: a stream
    capture therefore records them all.  Replays, with eager work in between, must reproduce the eager
    results bit for bit."""
    d = small_inputs(19, "bf16", 1, 2048, 4, 64, 1, 128)       # four segments of 512: several in flight
    dv = dev_inputs(d, "bf16")
    Q, seg = 256, 512
    shape = pk.make_shape(dv["x"], dv["B"], Q, seg)
    ws_f = torch.empty(pk.ssd_workspace_bytes(shape, False), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(pk.ssd_workspace_bytes(shape, True), dtype=torch.uint8, device="cuda")
    of = {"y": torch.empty_like(dv["x"]), "final_state": torch.empty((1, 4, 64, 128), device="cuda"),
          "boundary_states": torch.empty((1, 4, 4, 64, 128), device="cuda")}
    ob = {"dx": torch.empty_like(dv["x"]), "ddt": torch.empty_like(dv["dt"]), "dB": torch.empty_like(dv["B"]),
          "dC": torch.empty_like(dv["C"]), "dinit_state": torch.empty((1, 4, 64, 128), device="cuda")}
    dA, dD = torch.empty(4, device="cuda"), torch.empty(4, device="cuda")

    def step():
        pk.ssd_fwd(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], Q, seg, dv["init_state"], 0, ws_f, out=of)
        pk.ssd_bwd(dv["x"], dv["dt"], dv["A"], dv["B"], dv["C"], dv["D"], dv["dy"], Q, seg, dv["init_state"],
                   dv["dfinal_state"], of["boundary_states"], 0, ws_b, dA, dD, out=ob)

    step()                                    # eager: creates the library's streams and events
    torch.cuda.synchronize()
    want = {k: v.clone() for k, v in {**of, **ob, "dA": dA, "dD": dD}.items()}
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in list(of.values()) + list(ob.values()) + [dA, dD]:
            t.zero_()                         # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in {**of, **ob, "dA": dA, "dD": dD}.items():
            assert torch.equal(v, want[k]), (rep, k)
