"""GPU parity: forward and backward of the QLoRA linear layer against the fp64 CPU oracle.
Tolerance (from the benchmark spec): max|err| <= 2e-2 * rms(ref) per GEMM output."""
import numpy as np
import pytest
import torch

from gpu_util import bits_f64, dev_bf16, dev_f32, download_quant, host_bits, upload_quant

pytestmark = pytest.mark.gpu

TOL = 2e-2


def _check(got_bits, ref, tag, few_terms=False):
    """max|err| <= 2e-2 * rms(ref).  few_terms: the output is a sum of only a handful of products
    (adapter gradients at a few tokens), its distribution is heavy-tailed and the largest entries'
    own bf16 rounding can exceed 2e-2 * rms; such entries must then be within one bf16 step (2^-8
    relative, the bound tested below) of the reference instead.  Prints how many entries needed it."""
    got = bits_f64(got_bits).reshape(ref.shape)
    rms = np.sqrt((ref ** 2).mean())
    aerr = np.abs(got - ref)
    err = aerr.max()
    print(f"  {tag}: max|err|/rms = {err / rms if rms > 0 else 0.0:.4f}", flush=True)
    assert np.isfinite(got).all(), tag
    if few_terms:
        relaxed = int(np.count_nonzero(aerr > TOL * rms))
        if relaxed:
            print(f"  {tag}: {relaxed} of {aerr.size} entries beyond 2e-2 * rms, held to one bf16 step", flush=True)
        assert np.all(aerr <= np.maximum(TOL * rms, 2.0 ** -8 * np.abs(ref))), tag
        return
    assert err <= TOL * rms, f"{tag}: max|err| {err:.4g} > {TOL} * rms {rms:.4g}"


def _run_case(oracle, ql, L, tag, with_lora=True, rows=None):
    """Quantise on the GPU (bit-exact with the oracle by the quantise tests), then compare
    Y, dX, dL1, dL2 with the oracle evaluated on the oracle's own dequantised weights."""
    M, h, o, r, s = L["M"], L["h"], L["o"], L["r"], L["s"]
    q = oracle.nf4_quantize(L["W"])
    What = oracle.nf4_dequant(q)
    Wq = upload_quant(q)
    X, dY = dev_bf16(L["X"]), dev_bf16(L["dY"])
    L1 = dev_bf16(L["L1"]) if with_lora else None
    L2 = dev_bf16(L["L2"]) if with_lora else None
    hL1 = L["L1"] if with_lora else None
    hL2 = L["L2"] if with_lora else None
    print(f"case {tag}: M={M} h={h} o={o} r={r if with_lora else 0}", flush=True)
    T = torch.empty((M, 2 * r), dtype=torch.bfloat16, device="cuda") if with_lora else None
    Y = ql.qlora_linear_fwd(X, Wq, L1, L2, s, T_save=T)
    dX, dL1, dL2 = ql.qlora_linear_bwd(dY, X, Wq, L1, L2, s, T_saved=T)
    torch.cuda.synchronize()
    _check(host_bits(Y)[rows] if rows is not None else host_bits(Y),
           oracle.linear_fwd(L["X"], What, hL1, hL2, s, rows=rows), f"{tag} Y")
    _check(host_bits(dX)[rows] if rows is not None else host_bits(dX),
           oracle.linear_bwd_dx(L["dY"], What, hL1, hL2, s, rows=rows), f"{tag} dX")
    if with_lora:
        r1, r2 = oracle.linear_bwd_dl(L["dY"], L["X"], hL1, hL2, s)
        _check(host_bits(dL1), r1, f"{tag} dL1", few_terms=M < 64)
        _check(host_bits(dL2), r2, f"{tag} dL2", few_terms=M < 64)
        # gradient checkpointing: no saved T, recompute X L1 in the backward
        dXb, dL1b, dL2b = ql.qlora_linear_bwd(dY, X, Wq, L1, L2, s, T_saved=None)
        torch.cuda.synchronize()
        _check(host_bits(dL2b), r2, f"{tag} dL2 (recomputed T)", few_terms=M < 64)
        assert torch.equal(dXb, dX) and torch.equal(dL1b, dL1)
    return Y, dX


def test_no_adapter_small(oracle, synth):
    import paper_2305_14314_amd as ql
    L = synth.make_layer(0, 0)
    _run_case(oracle, ql, L, "config0 r=0", with_lora=False)


def test_no_adapter_ragged(oracle, synth):
    """M, o and h that are not multiples of the 256-wide tiles; several K steps."""
    import paper_2305_14314_amd as ql
    L = synth.make_layer(0, 0, M=300, h=448, o=576)
    _run_case(oracle, ql, L, "ragged r=0", with_lora=False)


def test_config0_full(oracle, synth):
    """Workload 0: 1024 x 1024, r = 16, alpha = 16, 256 tokens; every output element is checked."""
    import paper_2305_14314_amd as ql
    L = synth.make_layer(0, 0)
    _run_case(oracle, ql, L, "config0")


@pytest.mark.parametrize("M,h,o,r", [(300, 448, 576, 32), (1, 64, 64, 16), (17, 128, 320, 64), (513, 256, 192, 128),
                                      (64, 1024, 64, 256), (65, 64, 128, 16), (257, 64, 64, 64), (700, 192, 832, 48)])
def test_ragged_shapes(oracle, synth, M, h, o, r):
    """Token counts and feature sizes that do not fill the 256-wide tiles, several ranks; h = 64 is a single K-step
    of the large GEMM (shorter than its prefetch ring), o = 832 leaves a 64-column remainder in the last tile."""
    import paper_2305_14314_amd as ql
    L = synth.make_layer(0, 0, M=M, h=h, o=o, r=r)
    _run_case(oracle, ql, L, f"ragged M={M} h={h} o={o} r={r}")


def test_scalar_s_and_zero_adapter(oracle, synth):
    import paper_2305_14314_amd as ql
    L = synth.make_layer(0, 0, M=96, h=256, o=384, r=16)
    L["s"] = 0.0
    _run_case(oracle, ql, L, "s=0")
    L["s"] = 2.5                                            # not a power of two
    _run_case(oracle, ql, L, "s=2.5")
    L["L2"] = np.zeros_like(L["L2"])
    _run_case(oracle, ql, L, "L2=0")


def test_run_to_run_determinism(synth):
    import paper_2305_14314_amd as ql
    L = synth.make_layer(0, 0, M=200, h=512, o=448, r=16)
    Wq = ql.qlora_nf4_quantize(dev_f32(L["W"]))
    X, dY, L1, L2 = (dev_bf16(L[k]) for k in ("X", "dY", "L1", "L2"))
    a = ql.qlora_linear_fwd(X, Wq, L1, L2, L["s"])
    b = ql.qlora_linear_fwd(X, Wq, L1, L2, L["s"])
    ga = ql.qlora_linear_bwd(dY, X, Wq, L1, L2, L["s"])
    gb = ql.qlora_linear_bwd(dY, X, Wq, L1, L2, L["s"])
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    for u, v in zip(ga, gb):
        assert torch.equal(u, v)


@pytest.mark.parametrize("M,h,o,r", [(200, 512, 448, 16), (9, 320, 448, 64), (1024, 1024, 1024, 128)])
def test_gradient_accumulation(oracle, synth, M, h, o, r):
    """qlora_linear_bwd_acc over three micro-batches: the fp32 accumulators hold the sum of the oracle's three
    gradients.  No bf16 rounding is involved, so the bound is far below the output tolerance: the operands are exact
    bf16, T and U are carried with 16 significant bits (relative 2^-17 per product term) and the sums are fp32."""
    import paper_2305_14314_amd as ql
    s = 0.75
    W = synth.normal_f32((h, o), synth.SIGMA_W, 7000)
    q = oracle.nf4_quantize(W)
    Wq = upload_quant(q)
    hL1, hL2 = synth.normal_bf16((h, r), 0.05, 7001), synth.normal_bf16((r, o), 0.05, 7002)
    L1, L2 = dev_bf16(hL1), dev_bf16(hL2)
    a1 = torch.zeros((h, r), dtype=torch.float32, device="cuda")
    a2 = torch.zeros((r, o), dtype=torch.float32, device="cuda")
    r1 = np.zeros((h, r))
    r2 = np.zeros((r, o))
    dX_ref = None
    for mb in range(3):
        hX, hdY = synth.normal_bf16((M, h), 1.0, 7100 + mb), synth.normal_bf16((M, o), 1.0, 7200 + mb)
        X, dY = dev_bf16(hX), dev_bf16(hdY)
        T = torch.empty((M, 2 * r), dtype=torch.bfloat16, device="cuda") if mb != 1 else None   # one batch recomputes T
        if T is not None:
            ql.qlora_linear_fwd(X, Wq, L1, L2, s, T_save=T)
        dX = ql.qlora_linear_bwd_acc(dY, X, Wq, L1, L2, s, a1, a2, T_saved=T)
        dXb, _, _ = ql.qlora_linear_bwd(dY, X, Wq, L1, L2, s, T_saved=T)
        torch.cuda.synchronize()
        assert torch.equal(dX.view(torch.int16), dXb.view(torch.int16))      # dX does not depend on the variant
        g1, g2 = oracle.linear_bwd_dl(hdY, hX, hL1, hL2, s)
        r1 += g1
        r2 += g2
    for got, ref, tag in ((a1, r1, "dL1_acc"), (a2, r2, "dL2_acc")):
        got = got.cpu().numpy().astype(np.float64)
        rms = np.sqrt((ref ** 2).mean())
        err = np.abs(got - ref).max()
        print(f"  {tag}: max|err|/rms = {err / rms:.2e}", flush=True)
        assert err <= 2e-4 * rms, f"{tag}: max|err| {err:.3g} > 2e-4 * rms {rms:.3g}"


FULL = [(1, 0), (1, 4), (1, 6), (2, 0), (2, 4), (2, 6), (3, 0), (3, 4), (3, 6)]   # (config, layer): the distinct shapes


@pytest.mark.parametrize("config,layer", FULL)
def test_full_size_sampled(oracle, synth, config, layer):
    """LLaMA-shaped linears at the benchmark's token counts.  Y and dX are checked on sampled token rows
    (first/last rows of several 256-row tiles) and sampled columns; dL1/dL2 in full for the square shapes."""
    import paper_2305_14314_amd as ql
    cfg = synth.CONFIGS[config]
    h, o = cfg["linears"][layer]
    M, r, s = cfg["M"], cfg["r"], cfg["alpha"] / cfg["r"]
    print(f"case config{config} layer{layer}: M={M} h={h} o={o} r={r}", flush=True)
    Wd = synth.normal_f32_device((h, o), synth.SIGMA_W, synth.tensor_seed(config, layer, "W"))
    Wq = ql.qlora_nf4_quantize(Wd)
    del Wd
    q = download_quant(Wq)
    What = oracle.nf4_dequant(q)
    hX = synth.normal_bf16((M, h), 1.0, synth.tensor_seed(config, layer, "X"))
    hdY = synth.normal_bf16((M, o), 1.0, synth.tensor_seed(config, layer, "dY"))
    hL1 = synth.normal_bf16((h, r), cfg["sigma_l"], synth.tensor_seed(config, layer, "L1"))
    hL2 = synth.normal_bf16((r, o), cfg["sigma_l"], synth.tensor_seed(config, layer, "L2"))
    X, dY, L1, L2 = dev_bf16(hX), dev_bf16(hdY), dev_bf16(hL1), dev_bf16(hL2)
    T = torch.empty((M, 2 * r), dtype=torch.bfloat16, device="cuda")
    Y = ql.qlora_linear_fwd(X, Wq, L1, L2, s, T_save=T)
    dX, dL1, dL2 = ql.qlora_linear_bwd(dY, X, Wq, L1, L2, s, T_saved=T)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 1, 255, 256, 257, 511, 512, M // 2 - 1, M // 2, M - 257, M - 256, M - 1],
                                     np.random.default_rng(config * 10 + layer).integers(0, M, 20)])).astype(np.int64)
    _check(host_bits(Y)[rows], oracle.linear_fwd(hX, What, hL1, hL2, s, rows=rows), "Y rows")
    _check(host_bits(dX)[rows], oracle.linear_bwd_dx(hdY, What, hL1, hL2, s, rows=rows), "dX rows")
    ycols = np.array([0, 255, 256, o // 2 + 3, o - 256, o - 1], np.int64)
    xcols = np.array([0, 255, 256, h // 2 + 3, h - 256, h - 1], np.int64)
    _check(host_bits(Y)[:, ycols], oracle.linear_fwd(hX, What, hL1, hL2, s, cols=ycols), "Y cols")
    _check(host_bits(dX)[:, xcols], oracle.linear_bwd_dx(hdY, What, hL1, hL2, s, cols=xcols), "dX cols")
    if layer == 0 or (config, layer) == (3, 4):
        r1, r2 = oracle.linear_bwd_dl(hdY, hX, hL1, hL2, s)
        _check(host_bits(dL1), r1, "dL1")
        _check(host_bits(dL2), r2, "dL2")
    # the same input gradient with the weight decoded inside the product: same oracle rows and columns, and without
    # the adapter the same bits as the two-kernel form (the decoded tiles are identical)
    prev = ql.qlora_bwd_fused_dequant(1)
    try:
        dXf = ql.qlora_linear_bwd(dY, X, Wq, L1, L2, s, T_saved=T, need_dL=False)[0]
        dXf0 = ql.qlora_linear_bwd(dY, None, Wq, None, None, 0.0, need_dL=False)[0]
        ql.qlora_bwd_fused_dequant(0)
        dX0 = ql.qlora_linear_bwd(dY, None, Wq, None, None, 0.0, need_dL=False)[0]
        torch.cuda.synchronize()
    finally:
        ql.qlora_bwd_fused_dequant(prev)
    _check(host_bits(dXf)[rows], oracle.linear_bwd_dx(hdY, What, hL1, hL2, s, rows=rows), "dX rows (fused)")
    _check(host_bits(dXf)[:, xcols], oracle.linear_bwd_dx(hdY, What, hL1, hL2, s, cols=xcols), "dX cols (fused)")
    assert torch.equal(dXf0, dX0)


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        M = int(rng.choice([1, 2, 7, 15, 16, 17, 31, 64, 100, 255, 256, 257, 400, 600]))
        h = 64 * int(rng.integers(1, 25))
        o = 64 * int(rng.integers(1, 25))
        r = int(rng.choice([0, 16, 32, 48, 64, 80, 128, 256]))
        out.append((M, h, o, r))
    return out


@pytest.mark.parametrize("M,h,o,r", _random_shapes(24, 20240521))
def test_random_shapes(oracle, synth, M, h, o, r):
    """Seeded random token counts (both sides of the few-token threshold and of the 256-row tile), feature sizes
    (multiples of 64 up to 1536) and ranks: forward, input gradient and adapter gradients against the oracle."""
    import paper_2305_14314_amd as ql
    L = synth.make_layer(0, 0, M=M, h=h, o=o, r=max(r, 16))
    _run_case(oracle, ql, L, f"random M={M} h={h} o={o} r={r}", with_lora=r > 0)


def test_training_step_graph_replay(synth):
    """The large-GEMM path under HIP graph capture: forward with T saved, backward with all three gradients, the
    dropout variants with fp32 accumulation.  Every replay -- with eager work, scribbled workspace and synchronisations
    in between -- reproduces the eager result bit for bit (the path holds kernels only: nothing a graph replays badly)."""
    import paper_2305_14314_amd as ql
    M, h, o, r, s, p = 300, 448, 576, 32, 0.5, 0.1
    Wq = ql.qlora_nf4_quantize(synth.normal_f32_device((h, o), synth.SIGMA_W, 7100))
    L1 = dev_bf16(synth.normal_bf16((h, r), 0.05, 7101))
    L2 = dev_bf16(synth.normal_bf16((r, o), 0.05, 7102))
    X = dev_bf16(synth.normal_bf16((M, h), 1.0, 7103))
    dY = dev_bf16(synth.normal_bf16((M, o), 1.0, 7104))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7105)
    mask = ql.pack_keep_mask(torch.rand(M, h, device="cuda", generator=gen) >= p)
    nbytes = max(ql.qlora_linear_fwd_sizes(M, h, o, r), ql.qlora_linear_bwd_sizes(M, h, o, r),
                 *ql.qlora_linear_dropout_sizes(M, h, o, r))
    ws = ql.workspace_alloc(nbytes)
    hdr = ql.binding.WORKSPACE_HEADER_BYTES
    bufs = dict(Y=torch.empty(M, o, dtype=torch.bfloat16, device="cuda"), T=torch.empty(M, 2 * r, dtype=torch.bfloat16, device="cuda"),
                dX=torch.empty(M, h, dtype=torch.bfloat16, device="cuda"), dL1=torch.empty_like(L1), dL2=torch.empty_like(L2),
                Yd=torch.empty(M, o, dtype=torch.bfloat16, device="cuda"), dXd=torch.empty(M, h, dtype=torch.bfloat16, device="cuda"),
                a1=torch.zeros(h, r, dtype=torch.float32, device="cuda"), a2=torch.zeros(r, o, dtype=torch.float32, device="cuda"))

    def step():
        ql.qlora_linear_fwd(X, Wq, L1, L2, s, Y=bufs["Y"], T_save=bufs["T"], workspace=ws)
        ql.qlora_linear_bwd(dY, X, Wq, L1, L2, s, T_saved=bufs["T"], dX=bufs["dX"], dL1=bufs["dL1"], dL2=bufs["dL2"],
                            workspace=ws)
        ql.qlora_linear_fwd_dropout(X, Wq, L1, L2, s, mask, p, Y=bufs["Yd"], workspace=ws)
        ql.qlora_linear_bwd_dropout(dY, X, Wq, L1, L2, s, mask, p, dX=bufs["dXd"], dL1_acc=bufs["a1"], dL2_acc=bufs["a2"],
                                    workspace=ws)

    def clear():
        for k, t in bufs.items():
            t.zero_()

    clear()
    step()
    torch.cuda.synchronize()
    want = {k: t.clone() for k, t in bufs.items()}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for it in range(3):
        clear()
        ws[hdr:].random_(0, 255)                             # stale contents behind the counter header must not matter
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k, t in bufs.items():
            assert torch.equal(t.view(torch.int32 if t.dtype == torch.float32 else torch.int16),
                               want[k].view(torch.int32 if t.dtype == torch.float32 else torch.int16)), f"replay {it}: {k} differs"
        assert int(ws[:hdr].max()) == 0
