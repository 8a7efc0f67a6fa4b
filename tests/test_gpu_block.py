"""GPU parity of one whole Mamba-2 block under sequence checkpoints (forward, and the backward sweep that
recomputes every segment from its two states) against the fp64 block oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2411_19460_amd as pk
from oracle import block_ref
from paper_2411_19460_amd import synth
from parity_util import TOL, check, host

pytestmark = pytest.mark.gpu

BF = lambda a: np.asarray(synth.round_bf16(a), dtype=np.float64)
F32 = lambda a: np.asarray(a, dtype=np.float32).astype(np.float64)


def draw(seed, L, dm, H, P, G, N, pre=False):
    r = np.random.default_rng(4000 + seed)
    d_inner, conv_dim, d_in = block_ref.dims(None, H, P, G, N)
    dt0 = np.exp(r.uniform(np.log(1e-3), np.log(0.1), H))           # the step sizes the bias alone would give
    p = dict(W_in=BF(r.standard_normal((d_in, dm)) / np.sqrt(dm)), conv_w=F32(r.standard_normal((conv_dim, 4)) * 0.5),
             conv_b=F32(r.standard_normal(conv_dim) * 0.2), dt_bias=F32(dt0 + np.log(-np.expm1(-dt0))),
             A=F32(-np.exp(r.uniform(0.0, np.log(16.0), H))), D=F32(r.standard_normal(H)),
             norm_w=F32(1.0 + 0.3 * r.standard_normal(d_inner)), W_out=BF(r.standard_normal((dm, d_inner)) / np.sqrt(d_inner)))
    d = dict(u=BF(r.standard_normal((L, dm))), dout=BF(r.standard_normal((L, dm))), p=p)
    if pre:   # drawn last: the other values do not depend on it
        p["pre_norm_w"] = F32(1.0 + 0.3 * r.standard_normal(dm))
        d["u"] = BF(d["u"] * np.exp(r.uniform(-1.0, 1.0, (L, 1))))     # rows of different size: the normalisation has work to do
    return d


def to_dev(p):
    out = {}
    for k, v in p.items():
        t = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).cuda()
        out[k] = t.to(torch.bfloat16) if k in ("W_in", "W_out") else t
    return out


def dev_bf16(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(torch.bfloat16)


GRADS = ("dW_in", "dconv_w", "dconv_b", "ddt_bias", "dA", "dD", "dnorm_w", "dW_out")


@pytest.mark.parametrize("case", [
    # L,   d_model, H, P,  G, N,   chunk, segment
    (1024, 256, 8, 64, 1, 128, 128, 256),     # matrix-core scan kernels, four segments
    (700, 128, 8, 64, 2, 128, 256, 256),      # two groups; ragged: the last segment has 188 tokens
    (300, 64, 8, 16, 1, 16, 64, 128),         # small heads and states: the scan's shape-generic kernels
    (1536, 2560, 80, 64, 1, 128, 256, 1024),  # the 2.7B block at its real widths (10576-wide projection), 1.5 segments
    (517, 128, 8, 64, 1, 128, 128, 256),      # a last segment of five tokens: forward takes the generation kernels, backward recomputes it as a chunk
])
def test_block_forward_backward(case):
    L, dm, H, P, G, N, Q, seg = case
    d = draw(1, L, dm, H, P, G, N)
    u, dout, par = dev_bf16(d["u"]), dev_bf16(d["dout"]), to_dev(d["p"])
    f = pk.magc_block_fwd(u, par, H, P, G, N, Q, seg)
    g = pk.magc_block_bwd(u, par, dout, f["ssm_ckpt"], f["conv_ckpt"], H, P, G, N, Q, seg)
    torch.cuda.synchronize()
    fo = block_ref.block_fwd(d["u"], d["p"], H, P, G, N, 1e-5, store=synth.round_bf16)
    go = block_ref.block_bwd(d["u"], d["p"], H, P, G, N, d["dout"], 1e-5, store=synth.round_bf16)
    tol = TOL["bf16"]
    rep = {}
    check("out", host(f["out"]), fo["out"], tol, rep)
    check("final_ssm", host(f["final_ssm"]), fo["ssm_state"], tol, rep)
    check("final_conv", host(f["final_conv"]), fo["conv_state"], tol, rep)
    check("du", host(g["du"]), go["du"], tol, rep)
    for k in GRADS:
        check(k, host(g[k]), go[k], tol, rep)
    print("block errors:", {k: f"{v:.2e}" for k, v in rep.items()})
    # the checkpoint interval does not change the result (both states are carried exactly): one segment
    f1 = pk.magc_block_fwd(u, par, H, P, G, N, Q, None)
    g1 = pk.magc_block_bwd(u, par, dout, None, None, H, P, G, N, Q, None)
    torch.cuda.synchronize()
    assert torch.equal(f1["out"], f["out"])
    for k in ("du",) + GRADS:
        a, b = g[k].float(), g1[k].float()
        assert float((a - b).abs().max()) <= 2.0 ** -6 * float(b.abs().max()), k
    # accumulation into existing parameter gradients
    g2 = pk.magc_block_bwd(u, par, dout, f["ssm_ckpt"], f["conv_ckpt"], H, P, G, N, Q, seg, flags=pk.SSD_FLAG_ACCUM_PARAM,
                           grads={k: g[k].clone() for k in GRADS})
    torch.cuda.synchronize()
    for k in GRADS:
        check(k + " accumulated", host(g2[k]), 2 * host(g[k]), 1e-5)


@pytest.mark.parametrize("case", [
    (700, 128, 8, 64, 2, 128, 256, 256),      # ragged last segment
    (1536, 2560, 80, 64, 1, 128, 256, 1024),  # the 2.7B widths
])
def test_block_with_the_pre_norm(case):
    L, dm, H, P, G, N, Q, seg = case
    d = draw(6, L, dm, H, P, G, N, pre=True)
    u, dout, par = dev_bf16(d["u"]), dev_bf16(d["dout"]), to_dev(d["p"])
    f = pk.magc_block_fwd(u, par, H, P, G, N, Q, seg)
    g = pk.magc_block_bwd(u, par, dout, f["ssm_ckpt"], f["conv_ckpt"], H, P, G, N, Q, seg)
    torch.cuda.synchronize()
    fo = block_ref.block_fwd(d["u"], d["p"], H, P, G, N, 1e-5, store=synth.round_bf16)
    go = block_ref.block_bwd(d["u"], d["p"], H, P, G, N, d["dout"], 1e-5, store=synth.round_bf16)
    tol = TOL["bf16"]
    rep = {}
    check("out", host(f["out"]), fo["out"], tol, rep)
    check("du", host(g["du"]), go["du"], tol, rep)
    for k in GRADS + ("dpre_norm_w",):
        check(k, host(g[k]), go[k], tol, rep)
    print("pre-norm block errors:", {k: f"{v:.2e}" for k, v in rep.items()})
    # the parameter is what switches it on: without it the same call computes the plain block
    plain = {k: v for k, v in par.items() if k != "pre_norm_w"}
    f0 = pk.magc_block_fwd(u, plain, H, P, G, N, Q, seg)
    check("plain out", host(f0["out"]), block_ref.block_fwd(d["u"], {k: v for k, v in d["p"].items() if k != "pre_norm_w"},
                                                            H, P, G, N, 1e-5, store=synth.round_bf16)["out"], tol)
    # a missing gradient slot for it is refused before anything runs
    bad = {k: torch.empty_like(v) for k, v in g.items() if k in GRADS}
    with pytest.raises(pk.SSDError):
        pk.magc_block_bwd(u, par, dout, f["ssm_ckpt"], f["conv_ckpt"], H, P, G, N, Q, seg, grads=bad)


@pytest.mark.parametrize("variant", [(1, False), (2, True), (1, True)])
def test_block_prefill_then_generation_without_checkpoints(variant):
    # forward only: a prompt in segments with no checkpoint kept, then tokens one at a time (and three at
    # once) from the states the previous call left -- against the oracle run over the whole sequence
    G, pre = variant     # groups (two: the gated normalisation runs as a step of its own), with / without the pre-norm
    L0, dm, H, P, N, Q, seg = 600, 128, 8, 64, 128, 128, 256
    gen = [1, 1, 1, 3, 1, 16, 2]
    L = L0 + sum(gen)
    d = draw(3, L, dm, H, P, G, N, pre)
    u, par = dev_bf16(d["u"]), to_dev(d["p"])
    fo = block_ref.block_fwd(d["u"], d["p"], H, P, G, N, 1e-5, store=synth.round_bf16)
    f = pk.magc_block_fwd(u[:L0].contiguous(), par, H, P, G, N, Q, seg, checkpoints=False)
    assert f["ssm_ckpt"] is None
    tol = TOL["bf16"]
    check("prefill out", host(f["out"]), fo["out"][:L0], tol)
    # the same prompt with checkpoints gives the same output and states
    fc = pk.magc_block_fwd(u[:L0].contiguous(), par, H, P, G, N, Q, seg)
    assert torch.equal(fc["out"], f["out"]) and torch.equal(fc["final_ssm"], f["final_ssm"]) and torch.equal(fc["final_conv"], f["final_conv"])
    t, outs = L0, []
    for n in gen:
        f = pk.magc_block_fwd(u[t:t + n].contiguous(), par, H, P, G, N, Q, seg, init_ssm=f["final_ssm"], init_conv=f["final_conv"],
                              checkpoints=False)
        outs.append(f["out"])
        t += n
    torch.cuda.synchronize()
    check("generated out", host(torch.cat(outs)), fo["out"][L0:], tol)
    check("final ssm", host(f["final_ssm"]), fo["ssm_state"], tol)
    check("final conv", host(f["final_conv"]), fo["conv_state"], tol)


def test_block_state_adjoints_chain_two_calls():
    # a sequence cut in two by the caller: the second call starts from the first call's states, its state
    # adjoints feed the first call's backward -- together they are the whole sequence's gradients
    L, dm, H, P, G, N, Q, seg = 768, 128, 8, 64, 1, 128, 128, 256
    cut = 512
    d = draw(4, L, dm, H, P, G, N)
    u, dout, par = dev_bf16(d["u"]), dev_bf16(d["dout"]), to_dev(d["p"])
    ua, ub, da, db = (t.contiguous() for t in (u[:cut], u[cut:], dout[:cut], dout[cut:]))
    fa = pk.magc_block_fwd(ua, par, H, P, G, N, Q, seg)
    fb = pk.magc_block_fwd(ub, par, H, P, G, N, Q, seg, init_ssm=fa["final_ssm"], init_conv=fa["final_conv"])
    gb = pk.magc_block_bwd(ub, par, db, fb["ssm_ckpt"], fb["conv_ckpt"], H, P, G, N, Q, seg, init_ssm=fa["final_ssm"],
                           init_conv=fa["final_conv"], want_dinit=True)
    ga = pk.magc_block_bwd(ua, par, da, fa["ssm_ckpt"], fa["conv_ckpt"], H, P, G, N, Q, seg, dfinal_ssm=gb["dinit_ssm"],
                           dfinal_conv=gb["dinit_conv"], flags=pk.SSD_FLAG_ACCUM_PARAM, grads={k: gb[k] for k in GRADS})
    torch.cuda.synchronize()
    fo = block_ref.block_fwd(d["u"], d["p"], H, P, G, N, 1e-5, store=synth.round_bf16)
    go = block_ref.block_bwd(d["u"], d["p"], H, P, G, N, d["dout"], 1e-5, store=synth.round_bf16)
    tol = TOL["bf16"]
    check("out", host(torch.cat([fa["out"], fb["out"]])), fo["out"], tol)
    check("du", host(torch.cat([ga["du"], gb["du"]])), go["du"], tol)
    for k in GRADS:
        check(k, host(ga[k]), go[k], tol)


@pytest.mark.parametrize("case", [
    # layers, layer interval, L, segment      (d_model 128, 8 heads x 64, state 128, chunk 128)
    (3, 2, 640, 256),     # two layer groups (2 + 1), three segments, the last one short
    (4, 4, 512, 256),     # one layer group: only the stack input is kept on the layer axis
    (3, 1, 384, 384),     # every layer input kept, one segment
    (3, 2, 640, 256, True),   # the first grid again, every layer with its pre-norm: the language model's residual layer
])
def test_stack_of_blocks_on_the_two_axis_grid(case):
    NL, l, L, seg = case[:4]
    pre = len(case) > 4
    GRADS = globals()["GRADS"] + (("dpre_norm_w",) if pre else ())
    dm, H, P, G, N, Q = 128, 8, 64, 1, 128, 128
    ds = [draw(10 + j, L, dm, H, P, G, N, pre) for j in range(NL)]
    layers_h = [x["p"] for x in ds]
    x0h, douth = ds[0]["u"], ds[0]["dout"]
    x0, dout, layers = dev_bf16(x0h), dev_bf16(douth), [to_dev(p) for p in layers_h]
    f = pk.magc_blockstack_fwd(x0, layers, H, P, G, N, Q, seg, l)
    g = pk.magc_blockstack_bwd(x0, layers, dout, f["l_ckpt"], f["ssm_ckpt"], f["conv_ckpt"], H, P, G, N, Q, seg, l)
    torch.cuda.synchronize()
    fo = block_ref.stack_fwd(x0h, layers_h, H, P, G, N, 1e-5, store=synth.round_bf16)
    go = block_ref.stack_bwd(fo["xs"], layers_h, H, P, G, N, douth, 1e-5, store=synth.round_bf16)
    tol = 2 * TOL["bf16"]     # activations and their gradients are re-rounded to bf16 after every layer
    rep = {}
    check("out", host(f["out"]), fo["out"], tol, rep)
    check("dx0", host(g["dx0"]), go["dx0"], tol, rep)
    # Parameter gradients: fixed bars.  Largest errors seen on these four grids: ddt_bias of the lowest layer
    # 5.0e-2 (a sum over every token of terms that cancel, reached by a gradient that has crossed every layer
    # above: bar 3 TOL), dA 3.7e-2, dW_in 3.3e-2, everything else below 2.2e-2 (bar 2 TOL, as for out and dx0).
    for j in range(NL):
        for k in GRADS:
            check(f"layer {j} {k}", host(g["grads"][j][k]), go["grads"][j][k], 3 * TOL["bf16"] if k == "ddt_bias" else tol, rep)
    print("stack of blocks, worst errors:", {k: f"{v:.2e}" for k, v in sorted(rep.items(), key=lambda kv: -kv[1])[:4]})
    # the grid does not change the result: whole sequence as one segment, every layer input kept
    f1 = pk.magc_blockstack_fwd(x0, layers, H, P, G, N, Q, None, 1)
    g1 = pk.magc_blockstack_bwd(x0, layers, dout, f1["l_ckpt"], f1["ssm_ckpt"], f1["conv_ckpt"], H, P, G, N, Q, None, 1)
    torch.cuda.synchronize()
    assert torch.equal(f1["out"], f["out"])
    assert float((g1["dx0"].float() - g["dx0"].float()).abs().max()) <= 2.0 ** -6 * float(g1["dx0"].float().abs().max())
    for j in range(NL):
        for k in GRADS:
            a, b = g["grads"][j][k], g1["grads"][j][k]
            assert float((a - b).abs().max()) <= 2.0 ** -6 * float(b.abs().max()), (j, k)


@pytest.mark.parametrize("pre", [False, True])
def test_stack_inference_prompt_then_tokens(pre):
    # forward only, nothing kept: a prompt in segments (the last one short), then tokens one at a time and three
    # at once, every call continuing from the per-layer states the previous one left -- against the oracle run
    # over the whole sequence, outputs and the states of every layer
    NL, L0, seg, gen = 3, 600, 256, [1, 1, 3, 1]
    dm, H, P, G, N, Q = 128, 8, 64, 1, 128, 128
    L = L0 + sum(gen)
    ds = [draw(20 + j, L, dm, H, P, G, N, pre) for j in range(NL)]
    layers_h, x0h = [x["p"] for x in ds], ds[0]["u"]
    x0, layers = dev_bf16(x0h), [to_dev(p) for p in layers_h]
    fo = block_ref.stack_fwd(x0h, layers_h, H, P, G, N, 1e-5, store=synth.round_bf16)
    st = pk.magc_blockstack_infer(x0[:L0].contiguous(), layers, H, P, G, N, Q, seg)
    # the training forward pass computes the same thing for the prompt
    ft = pk.magc_blockstack_fwd(x0[:L0].contiguous(), layers, H, P, G, N, Q, seg, 2)
    assert torch.equal(ft["out"], st["out"])
    outs, t = [st["out"]], L0
    for n in gen:
        xin = x0[t:t + n].clone()
        st = pk.magc_blockstack_infer(xin, layers, H, P, G, N, Q, seg, ssm_state=st["ssm_state"], conv_state=st["conv_state"],
                                      out=xin, workspace=st["workspace"])      # output over the input
        outs.append(st["out"])
        t += n
    torch.cuda.synchronize()
    tol = 2 * TOL["bf16"]
    check("out", host(torch.cat(outs)), fo["out"], tol)
    for j in range(NL):
        check(f"layer {j} ssm state", host(st["ssm_state"][j]), fo["ssm_states"][j], tol)
        check(f"layer {j} conv state", host(st["conv_state"][j]), fo["conv_states"][j], tol)


@pytest.mark.parametrize("shape", [(128, 8, 64, 2, 128, 128), (64, 8, 16, 1, 16, 64), (64, 8, 20, 4, 24, 64)])
def test_stack_generation_from_the_first_token(shape):
    # a new sequence that starts with calls of a few tokens: the first call has no state to read (zeros), its
    # convolution window reaches before the sequence; small and odd head and state sizes (rows of the state that
    # do not fill a wave, heads that do not fill a workgroup), several groups
    dm, H, P, G, N, Q = shape
    NL, calls = 2, [2, 1, 5, 16, 1]
    L = sum(calls)
    ds = [draw(30 + j, L, dm, H, P, G, N, True) for j in range(NL)]
    layers_h, x0h = [x["p"] for x in ds], ds[0]["u"]
    x0, layers = dev_bf16(x0h), [to_dev(p) for p in layers_h]
    fo = block_ref.stack_fwd(x0h, layers_h, H, P, G, N, 1e-5, store=synth.round_bf16)
    st, outs, t = {}, [], 0
    for n in calls:
        st = pk.magc_blockstack_infer(x0[t:t + n].contiguous(), layers, H, P, G, N, Q, 4 * Q, ssm_state=st.get("ssm_state"),
                                      conv_state=st.get("conv_state"), workspace=st.get("workspace"))
        outs.append(st["out"])
        t += n
    torch.cuda.synchronize()
    tol = 2 * TOL["bf16"]
    check("out", host(torch.cat(outs)), fo["out"], tol)
    for j in range(NL):
        check(f"layer {j} ssm state", host(st["ssm_state"][j]), fo["ssm_states"][j], tol)
        check(f"layer {j} conv state", host(st["conv_state"][j]), fo["conv_states"][j], tol)


@pytest.mark.parametrize("shape", [(128, 8, 64, 1, 128, 128, True, 5), (128, 8, 64, 2, 128, 128, False, 16), (64, 8, 16, 1, 16, 64, True, 3),
                                   (64, 8, 16, 1, 16, 4, True, 16)])     # more sequences than a segment has rows: sequence by sequence
def test_stack_generation_for_several_sequences_at_once(shape):
    # sequences of different lengths, each prefilled on its own, then generated together one token per step:
    # every sequence against the oracle run over that sequence alone (sixteen sequences of the wide-state shape:
    # more convolution state than the last launch can move on the side, so it is copied per sequence)
    dm, H, P, G, N, Q, pre, nseq = shape
    NL, steps = 2, 3
    lens = [70, 1, 300, 33, 150, 2, 5, 64, 129, 17, 3, 40, 90, 8, 256, 11][:nseq]
    seg = 2 * Q
    d_inner, conv_dim, _ = block_ref.dims(None, H, P, G, N)
    base = [draw(40 + j, max(lens) + steps, dm, H, P, G, N, pre) for j in range(NL)]
    layers_h = [x["p"] for x in base]
    layers = [to_dev(p) for p in layers_h]
    r = np.random.default_rng(77)
    seqs_h = [BF(r.standard_normal((n + steps, dm)) * np.exp(r.uniform(-1.0, 1.0, (n + steps, 1)))) for n in lens]
    ssm = torch.zeros((nseq, NL, H, P, N), dtype=torch.float32, device="cuda")
    conv = torch.zeros((nseq, NL, 3, conv_dim), dtype=torch.bfloat16, device="cuda")
    for i, n in enumerate(lens):     # prefill writes each sequence's slice of the two state arrays
        xi = dev_bf16(seqs_h[i][:n])
        st = pk.magc_blockstack_infer(xi, layers, H, P, G, N, Q, seg)
        ssm[i].copy_(st["ssm_state"])
        conv[i].copy_(st["conv_state"])
    outs, ws = [], None
    for t in range(steps):
        x = dev_bf16(np.stack([seqs_h[i][lens[i] + t] for i in range(nseq)]))
        o = pk.magc_blockstack_decode(x, layers, H, P, G, N, Q, seg, ssm, conv, workspace=ws)
        ws = o["workspace"]
        outs.append(o["out"])
    torch.cuda.synchronize()
    tol = 2 * TOL["bf16"]
    for i, n in enumerate(lens):
        fo = block_ref.stack_fwd(seqs_h[i], layers_h, H, P, G, N, 1e-5, store=synth.round_bf16)
        got = torch.stack([outs[t][i] for t in range(steps)])
        check(f"sequence {i} generated", host(got), fo["out"][n:], tol)
        for j in range(NL):
            check(f"sequence {i} layer {j} ssm state", host(ssm[i, j]), fo["ssm_states"][j], tol)
            check(f"sequence {i} layer {j} conv state", host(conv[i, j]), fo["conv_states"][j], tol)


def test_generation_step_replays_as_a_graph():
    """A generation step enqueues kernels only (no memset, no allocation with buffers given, one stream): captured
    once, each replay advances the sequence by the token in the static input buffer exactly as an eager call does."""
    NL, L0, ngen = 2, 100, 4
    dm, H, P, G, N, Q, seg = 128, 8, 64, 1, 128, 128, 256
    ds = [draw(50 + j, L0 + ngen, dm, H, P, G, N, True) for j in range(NL)]
    layers = [to_dev(x["p"]) for x in ds]
    x = dev_bf16(ds[0]["u"])
    st = pk.magc_blockstack_infer(x[:L0].contiguous(), layers, H, P, G, N, Q, seg)
    ssm0, conv0 = st["ssm_state"].clone(), st["conv_state"].clone()
    # eager reference: one call per token from copies of the states
    ssm, conv, want, ws = ssm0.clone(), conv0.clone(), [], None
    for t in range(ngen):
        o = pk.magc_blockstack_infer(x[L0 + t:L0 + t + 1].contiguous(), layers, H, P, G, N, Q, seg, ssm_state=ssm, conv_state=conv, workspace=ws)
        ws = o["workspace"]
        want.append(o["out"].clone())
    torch.cuda.synchronize()
    want_ssm, want_conv = ssm.clone(), conv.clone()
    # the same step captured once on static buffers
    ssm.copy_(ssm0)
    conv.copy_(conv0)
    tok, out = torch.empty((1, dm), dtype=torch.bfloat16, device="cuda"), torch.empty((1, dm), dtype=torch.bfloat16, device="cuda")
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            pk.magc_blockstack_infer(tok, layers, H, P, G, N, Q, seg, ssm_state=ssm, conv_state=conv, out=out, workspace=ws)
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 16, device="cuda")
    for t in range(ngen):
        tok.copy_(x[L0 + t:L0 + t + 1])
        scratch.add_(1.0)                     # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want[t]), t
    assert torch.equal(ssm, want_ssm) and torch.equal(conv, want_conv)


def test_block_rejects_bad_shapes():
    u = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    d = draw(2, 64, 64, 4, 16, 1, 16)       # four heads: the projection's width is not a multiple of 8
    with pytest.raises(pk.SSDError):
        pk.magc_block_fwd(u, to_dev(d["p"]), 4, 16, 1, 16, 64, 64)
