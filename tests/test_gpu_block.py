"""GPU parity of the decoder-block launcher and the model wrapper against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import forge_oracle as O
from paper_2604_16498_amd import inputs as I
from util import check, check_drift, dev, dev_dict, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def F():
    from paper_2604_16498_amd import binding
    binding.lib()
    return binding


def run_block(F, sh, w, x, bf16, cap, pos0=0, kc=None, vc=None):
    """One layer on the GPU; returns (x_out, k_cache, v_cache) tensors."""
    B, S, _ = x.shape
    dt = torch.bfloat16 if bf16 else torch.float32
    tw = dev_dict(w, bf16)
    desc = F.make_block_desc(sh, tw)
    tx = dev(x, bf16)
    out = torch.empty_like(tx)
    tk = torch.zeros(B, sh.kv_heads, cap, sh.head_dim, dtype=dt, device="cuda") if kc is None else kc
    tv = torch.zeros_like(tk) if vc is None else vc
    ws = F.workspace(F.forge_decoder_block_workspace_bytes(desc, B, S, cap))
    F.forge_decoder_block(desc, tx, out, tk, tv, pos0, ws)
    torch.cuda.synchronize()
    return out, tk, tv


def test_config1_gpt2_layer_fp32(F):
    """Configuration 1 in full: one GPT-2-small layer, fp32, batch 1, 128 tokens."""
    wl = I.WORKLOADS[1]
    sh = wl.block
    w = I.block_weights(sh, 1, 0, bf16=False, bias_std=0.0)
    x = I.hidden_states(wl)
    ref = O.decoder_block(sh, w, x)
    out, tk, tv = run_block(F, sh, w, x, False, cap=128)
    err = check(out, ref, False, "config 1 block")
    print("config1 max-abs err %.3e" % err)
    # bitwise reproducible
    out2, _, _ = run_block(F, sh, w, x, False, cap=128)
    assert torch.equal(out, out2)


SMALL_GPT = I.BlockShape(256, 4, 4, 64, 1024)
SMALL_LLAMA = I.BlockShape(512, 8, 2, 64, 704, norm="rmsnorm", mlp_act="swiglu", use_rope=True,
                           rope_base=500000.0, has_bias=False)
SMALL_LLAMA128 = I.BlockShape(512, 4, 1, 128, 1408, norm="rmsnorm", mlp_act="swiglu", use_rope=True,
                              rope_base=500000.0, has_bias=False)


SMALL_GPT_ERF = I.BlockShape(256, 4, 4, 64, 1024, mlp_act="gelu_erf")


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("sh", [SMALL_GPT, SMALL_LLAMA, SMALL_LLAMA128, SMALL_GPT_ERF],
                         ids=["gpt", "llama64", "llama128", "gpt-erf-gelu"])
def test_block_prefill_then_decode(F, sh, bf16):
    B, S, cap = 2, 150, 160
    w = I.block_weights(sh, 70, 0, bf16=bf16, bias_std=0.05, random_affine=True, weight_std=0.04)
    x = I.normal(70, 0, "x", (B, S + 1, sh.d_model), 1.0, bf16=bf16)
    kc = np.zeros((B, sh.kv_heads, cap, sh.head_dim)); vc = np.zeros_like(kc)
    ref = O.decoder_block(sh, w, x[:, :S], kc, vc, pos0=0)
    out, tk, tv = run_block(F, sh, w, x[:, :S], bf16, cap)
    check(out, ref, bf16, "prefill block", chain=True)
    check(tk, kc, bf16, "k cache"); check(tv, vc, bf16, "v cache")
    # decode step on the GPU's own cache; the oracle continues from its own
    ref1 = O.decoder_block(sh, w, x[:, S:], kc, vc, pos0=S)
    out1, tk, tv = run_block(F, sh, w, x[:, S:], bf16, cap, pos0=S, kc=tk, vc=tv)
    check(out1, ref1, bf16, "decode block", chain=True)
    check(tk, kc, bf16, "k cache after decode")


def test_block_decode_in_a_cache_sized_for_a_longer_generation(F):
    """A decode step at position 768 of a cache with room for 2049 rows, batch 8 over 8 KV heads
    (64 pairs: the split-KV attention cuts the 769 rows into MORE ranges than it would cut 2049).
    The layer's workspace, sized once for the capacity, must serve this step too."""
    sh = I.BlockShape(512, 32, 8, 64, 256, norm="rmsnorm", mlp_act="swiglu", use_rope=True,
                      rope_base=500000.0, has_bias=False)
    B, cap, pos0 = 8, 2049, 768
    w = I.block_weights(sh, 76, 0, bf16=True, random_affine=True, weight_std=0.04)
    x = I.normal(76, 0, "x", (B, 1, sh.d_model), 1.0, bf16=True)
    kc = np.zeros((B, sh.kv_heads, cap, sh.head_dim)); vc = np.zeros_like(kc)
    kc[:, :, :pos0] = I.normal(76, 0, "k_cache", (B, sh.kv_heads, pos0, sh.head_dim), 1.0, bf16=True)
    vc[:, :, :pos0] = I.normal(76, 0, "v_cache", (B, sh.kv_heads, pos0, sh.head_dim), 1.0, bf16=True)
    tk, tv = dev(kc.astype(np.float32), True), dev(vc.astype(np.float32), True)
    ref = O.decoder_block(sh, w, x, kc, vc, pos0=pos0)
    out, tk, tv = run_block(F, sh, w, x, True, cap, pos0=pos0, kc=tk, vc=tv)
    check(out, ref, True, "decode block at position 768 of 2049", chain=True)
    check(tk[:, :, :pos0 + 1], kc[:, :, :pos0 + 1], True, "k cache")
    # and through the attention call alone, with the scratch sized for the capacity
    q = I.normal(76, 1, "q", (B, sh.q_heads, 1, sh.head_dim), 1.0, bf16=True)
    ws = F.workspace(F.forge_attn_fused_workspace_bytes(B, sh.q_heads, sh.kv_heads, 1, cap, sh.head_dim, torch.bfloat16))
    o = torch.empty(B, 1, sh.q_heads * sh.head_dim, dtype=torch.bfloat16, device="cuda")
    F.forge_attn_fused(dev(q, True), tk, tv, o, pos0 + 1, causal=True, workspace=ws)
    torch.cuda.synchronize()
    check(o, O.attention(q, host(tk)[:, :, :pos0 + 1], host(tv)[:, :, :pos0 + 1], sh.head_dim ** -0.5, True), True,
          "attention over 769 of 2049 rows")


@pytest.mark.parametrize("flavour", ["gpt", "llama"])
def test_block_many_short_sequences(F, flavour):
    """400 sequences of 96 tokens: the QKV GEMM has more 128-row tiles (600) than resident blocks,
    and every tile spans two sequences, so the head split of the persistent kernel resolves
    (sequence, position) across tile rows and across the tiles one block walks over."""
    if flavour == "gpt":
        sh = I.BlockShape(128, 2, 1, 64, 128)
    else:
        sh = I.BlockShape(128, 2, 1, 64, 192, norm="rmsnorm", mlp_act="swiglu", use_rope=True,
                          rope_base=500000.0, has_bias=False)
    B, S = 400, 96
    w = I.block_weights(sh, 75, 0, bf16=True, bias_std=0.05, random_affine=True, weight_std=0.06)
    x = I.normal(75, 0, "x", (B, S, sh.d_model), 1.0, bf16=True)
    kc = np.zeros((B, sh.kv_heads, S, sh.head_dim)); vc = np.zeros_like(kc)
    ref = O.decoder_block(sh, w, x, kc, vc, pos0=0)
    out, tk, tv = run_block(F, sh, w, x, True, S)
    check(tk, kc, True, "k cache"); check(tv, vc, True, "v cache")
    check(out, ref, True, "block, many short sequences", chain=True)


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
def test_block_in_place(F, bf16):
    sh = SMALL_GPT
    w = I.block_weights(sh, 71, 0, bf16=bf16)
    x = I.normal(71, 0, "x", (1, 70, sh.d_model), 1.0, bf16=bf16)
    ref = O.decoder_block(sh, w, x)
    tw = dev_dict(w, bf16)
    desc = F.make_block_desc(sh, tw)
    tx = dev(x, bf16)
    tk = torch.zeros(1, sh.kv_heads, 70, sh.head_dim, dtype=tx.dtype, device="cuda"); tv = torch.zeros_like(tk)
    ws = F.workspace(F.forge_decoder_block_workspace_bytes(desc, 1, 70, 70))
    F.forge_decoder_block(desc, tx, tx, tk, tv, 0, ws)
    torch.cuda.synchronize()
    check(tx, ref, bf16, "in-place block", chain=True)


def test_block_rejects_small_workspace(F):
    sh = SMALL_GPT
    tw = dev_dict(I.block_weights(sh, 71, 0, bf16=True), True)
    desc = F.make_block_desc(sh, tw)
    tx = torch.zeros(1, 8, sh.d_model, dtype=torch.bfloat16, device="cuda")
    tk = torch.zeros(1, sh.kv_heads, 8, sh.head_dim, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(F.ForgeError) as e:
        F.forge_decoder_block(desc, tx, tx, tk, tk.clone(), 0, F.workspace(256))
    assert e.value.status == 3


@pytest.mark.parametrize("ld", [0, 1008], ids=["dense", "padded"])
@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
def test_model_forward_tokens(F, bf16, ld):
    """Small GPT-shaped model with embedding and tied head, odd vocabulary size; logits rows
    dense or padded to a 16-byte aligned stride."""
    sh = SMALL_GPT
    L, B, S, V = 3, 2, 90, 1001
    wl = I.scaled(I.WORKLOADS[2], block=sh, layers=L, vocab=V, n_pos=128, batch=B, seq=S, bf16=bf16)
    mw = I.model_weights(wl, random_affine=True)
    layers = [I.block_weights(sh, 72, l, bf16=bf16, random_affine=True) for l in range(L)]
    ids = I.token_ids(72, B, S, V)
    ref = O.gpt_forward(sh, layers, mw, ids=ids)
    dt = torch.bfloat16 if bf16 else torch.float32
    tl = [dev_dict(w, bf16) for w in layers]
    tm = dev_dict(mw, bf16)
    model = F.make_model_desc([F.make_block_desc(sh, w) for w in tl], tm, logits_ld=ld)
    full = torch.zeros(B, S, ld if ld else V, dtype=dt, device="cuda")
    logits = full[..., :V]
    kc = torch.zeros(L, B, sh.kv_heads, S, sh.head_dim, dtype=dt, device="cuda"); vc = torch.zeros_like(kc)
    ws = F.workspace(F.forge_model_workspace_bytes(model, B, S, S))
    F.forge_model_forward(model, torch.from_numpy(ids).cuda(), full, kc, vc, 0, ws)
    torch.cuda.synchronize()
    assert torch.all(full[..., V:] == 0)
    if bf16:
        check_drift(logits, ref, "model bf16, %d layers end to end" % L)
    else:
        check(logits, ref, False, "model logits")
    a = full.clone()
    F.forge_model_forward(model, torch.from_numpy(ids).cuda(), full, kc, vc, 0, ws)
    torch.cuda.synchronize()
    assert torch.equal(a, full)


def test_model_forward_hidden_llama(F):
    sh = SMALL_LLAMA128
    L, B, S = 2, 1, 130
    wl = I.scaled(I.WORKLOADS[4], block=sh, layers=L, batch=B, seq=S)
    mw = I.model_weights(wl, random_affine=True)
    layers = [I.block_weights(sh, 73, l, bf16=True, random_affine=True) for l in range(L)]
    x = I.hidden_states(wl)
    ref = O.gpt_forward(sh, layers, mw, x=x)
    tl = [dev_dict(w, True) for w in layers]
    tm = dev_dict(mw, True)
    model = F.make_model_desc([F.make_block_desc(sh, w) for w in tl], tm)
    out = torch.empty(B, S, sh.d_model, dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros(L, B, sh.kv_heads, S, sh.head_dim, dtype=torch.bfloat16, device="cuda"); vc = torch.zeros_like(kc)
    ws = F.workspace(F.forge_model_workspace_bytes(model, B, S, S))
    F.forge_model_forward(model, dev(x, True), out, kc, vc, 0, ws)
    torch.cuda.synchronize()
    check_drift(out, ref, "llama hidden states, %d layers end to end" % L)


@pytest.mark.parametrize("sh_name", ["llama", "gpt"])
def test_model_decode_step_hidden_state_stack(F, sh_name):
    """One decode step of a 3-layer stack fed with hidden states (no token table), against the
    oracle's layers applied one after the other on the same caches.  In a bf16 step of at most 64
    rows every norm after the first is produced by the reduce step of the projection before it
    (the second norm by the output projection, the next layer's first norm and the final norm by
    the MLP down projection), and the final norm lands in the caller's output."""
    sh = SMALL_LLAMA if sh_name == "llama" else SMALL_GPT
    L, B, cap, pos0 = 3, 5, 100, 70
    wl = I.scaled(I.WORKLOADS[4], block=sh, layers=L, batch=B, seq=1)
    mw = I.model_weights(wl, random_affine=True)
    layers = [I.block_weights(sh, 79, l, bf16=True, random_affine=True, weight_std=0.05) for l in range(L)]
    x = I.normal(79, 0, "x", (B, 1, sh.d_model), 1.0, bf16=True)
    kc = I.normal(79, 0, "k_cache", (L, B, sh.kv_heads, cap, sh.head_dim), 1.0, bf16=True)
    vc = I.normal(79, 0, "v_cache", (L, B, sh.kv_heads, cap, sh.head_dim), 1.0, bf16=True)
    h = x.astype(np.float64)
    for l in range(L):
        h = O.decoder_block(sh, layers[l], h, kc[l].astype(np.float64), vc[l].astype(np.float64), pos0=pos0)
    _, ref = O.residual_norm(h, None, mw["normf_g"], mw.get("normf_b"), sh.eps, sh.norm)
    tl = [dev_dict(w, True) for w in layers]
    tm = dev_dict(mw, True)
    model = F.make_model_desc([F.make_block_desc(sh, w) for w in tl], tm)
    out = torch.empty(B, 1, sh.d_model, dtype=torch.bfloat16, device="cuda")
    tk, tv = dev(kc, True), dev(vc, True)
    ws = F.workspace(F.forge_model_workspace_bytes(model, B, 1, cap))
    F.forge_model_forward(model, dev(x, True), out, tk, tv, pos0, ws)
    torch.cuda.synchronize()
    check_drift(out, ref, "%s decode stack, %d layers" % (sh_name, L))
    # per-sequence positions: the same step through forge_model_decode
    out2 = torch.empty_like(out)
    tk2, tv2 = dev(kc, True), dev(vc, True)
    F.forge_model_decode(model, dev(x, True), out2, tk2, tv2, torch.full((B,), pos0, dtype=torch.int32, device="cuda"), pos0, ws)
    torch.cuda.synchronize()
    assert torch.equal(out2, out) and torch.equal(tk2, tk) and torch.equal(tv2, tv)


def test_block_wide_model_short_prompt(F):
    """A 100-token prompt through a wide layer (d_model 1024, MLP 4096): every projection has few
    output tiles and a long reduction, i.e. the k-split path of the tile kernel, including the
    head split of the QKV projection."""
    sh = I.BlockShape(1024, 4, 2, 64, 4096, norm="rmsnorm", mlp_act="swiglu", use_rope=True,
                      rope_base=500000.0, has_bias=False)
    B, S = 1, 100
    w = I.block_weights(sh, 78, 0, bf16=True, random_affine=True, weight_std=0.03)
    x = I.normal(78, 0, "x", (B, S, sh.d_model), 1.0, bf16=True)
    kc = np.zeros((B, sh.kv_heads, S, sh.head_dim)); vc = np.zeros_like(kc)
    ref = O.decoder_block(sh, w, x, kc, vc, pos0=0)
    out, tk, tv = run_block(F, sh, w, x, True, S)
    check(tk, kc, True, "k cache"); check(tv, vc, True, "v cache")
    check(out, ref, True, "wide block, short prompt", chain=True)


def _random_block_cases():
    rng = np.random.default_rng(16498)
    cases = []
    for _ in range(12):
        dh = int(rng.choice([64, 128]))
        hkv = int(rng.choice([1, 2, 4]))
        hq = hkv * int(rng.choice([1, 2, 4]))
        d = int(rng.choice([128, 192, 256, 512]))
        ff = int(rng.choice([128, 264, 512, 1032]))
        llama = bool(rng.integers(2))
        B = int(rng.integers(1, 6)); S = int(rng.choice([1, 5, 31, 64, 100, 129, 257]))
        pos0 = int(rng.choice([0, 0, 3, 70]))
        cases.append((d, hq, hkv, dh, ff, llama, B, S, pos0))
    return cases


@pytest.mark.parametrize("d,hq,hkv,dh,ff,llama,B,S,pos0", _random_block_cases())
def test_block_random_shapes(F, d, hq, hkv, dh, ff, llama, B, S, pos0):
    """Seeded sweep over layer shapes: head counts and grouping, head_dim, widths that are not
    tile multiples, sequence lengths around the tile sizes, with and without cached positions."""
    if llama:
        sh = I.BlockShape(d, hq, hkv, dh, ff, norm="rmsnorm", mlp_act="swiglu", use_rope=True,
                          rope_base=10000.0, has_bias=False)
    else:
        sh = I.BlockShape(d, hq, hkv, dh, ff)
    cap = pos0 + S + 3
    w = I.block_weights(sh, 80, 0, bf16=True, bias_std=0.05, random_affine=True, weight_std=0.05)
    x = I.normal(80, 0, "x", (B, S, sh.d_model), 1.0, bf16=True)
    kc = np.zeros((B, sh.kv_heads, cap, sh.head_dim)); vc = np.zeros_like(kc)
    if pos0:
        kc[:, :, :pos0] = I.normal(80, 0, "k_cache", (B, sh.kv_heads, pos0, sh.head_dim), 1.0, bf16=True)
        vc[:, :, :pos0] = I.normal(80, 0, "v_cache", (B, sh.kv_heads, pos0, sh.head_dim), 1.0, bf16=True)
    tk, tv = dev(kc.astype(np.float32), True), dev(vc.astype(np.float32), True)
    ref = O.decoder_block(sh, w, x, kc, vc, pos0=pos0)
    out, tk, tv = run_block(F, sh, w, x, True, cap, pos0=pos0, kc=tk, vc=tv)
    check(out, ref, True, "block", chain=True)
    check(tk[:, :, :pos0 + S], kc[:, :, :pos0 + S], True, "k cache")
    check(tv[:, :, :pos0 + S], vc[:, :, :pos0 + S], True, "v cache")


def test_model_generation_loop(F):
    """Prefill of 24 tokens, then 8 single-token steps on the growing KV cache (teacher-forced
    ids): the logits of step i equal row 24 + i of one causal forward over all 32 tokens, which
    is what the oracle computes."""
    sh = SMALL_GPT
    L, B, S0, steps, V = 2, 3, 24, 8, 520
    cap = 64
    wl = I.scaled(I.WORKLOADS[2], block=sh, layers=L, vocab=V, n_pos=64, batch=B, seq=S0 + steps, bf16=True)
    mw = I.model_weights(wl, random_affine=True)
    layers = [I.block_weights(sh, 77, l, bf16=True, random_affine=True) for l in range(L)]
    ids = I.token_ids(77, B, S0 + steps, V)
    ref = O.gpt_forward(sh, layers, mw, ids=ids)                     # [B, S0 + steps, V]
    tl = [dev_dict(w, True) for w in layers]
    tm = dev_dict(mw, True)
    model = F.make_model_desc([F.make_block_desc(sh, w) for w in tl], tm)
    kc = torch.zeros(L, B, sh.kv_heads, cap, sh.head_dim, dtype=torch.bfloat16, device="cuda"); vc = torch.zeros_like(kc)
    tids = torch.from_numpy(ids).cuda()
    logits = torch.empty(B, S0, V, dtype=torch.bfloat16, device="cuda")
    ws = F.workspace(max(F.forge_model_workspace_bytes(model, B, S0, cap), F.forge_model_workspace_bytes(model, B, 1, cap)))
    F.forge_model_forward(model, tids[:, :S0].contiguous(), logits, kc, vc, 0, ws)
    torch.cuda.synchronize()
    check_drift(logits, ref[:, :S0], "generation loop, prompt")
    step_logits = torch.empty(B, 1, V, dtype=torch.bfloat16, device="cuda")
    worst = 0.0
    for i in range(steps):
        F.forge_model_forward(model, tids[:, S0 + i:S0 + i + 1].contiguous(), step_logits, kc, vc, S0 + i, ws)
        torch.cuda.synchronize()
        _, l2 = check_drift(step_logits, ref[:, S0 + i:S0 + i + 1], "generation loop, decode step %d" % i)
        worst = max(worst, l2)
    print("generation loop: worst l2 over %d steps %.3e" % (steps, worst))


@pytest.mark.parametrize("decode", [False, True], ids=["prefill", "decode"])
def test_block_under_hip_graph_capture(F, decode):
    """The launch list allocates nothing and never synchronises (Sec. "Code Generation:
    CompiledNPUExecutor": pre-resolved callables, no run-time allocation, fixed order), so a caller
    can capture it into a HIP graph.  Every replay, with eager work and synchronisations in
    between, must reproduce the eager result bit for bit."""
    sh = SMALL_LLAMA
    B, S, cap = (4, 1, 96) if decode else (2, 80, 96)
    pos0 = 64 if decode else 0
    w = I.block_weights(sh, 76, 0, bf16=True, weight_std=0.05)
    tw = dev_dict(w, True)
    desc = F.make_block_desc(sh, tw)
    x = dev(I.normal(76, 0, "x", (B, S, sh.d_model), 1.0, bf16=True), True)
    kc0 = dev(I.normal(76, 0, "k_cache", (B, sh.kv_heads, cap, sh.head_dim), 1.0, bf16=True), True)
    vc0 = dev(I.normal(76, 0, "v_cache", (B, sh.kv_heads, cap, sh.head_dim), 1.0, bf16=True), True)
    ws = F.workspace(F.forge_decoder_block_workspace_bytes(desc, B, S, cap))

    def fresh():
        return kc0.clone(), vc0.clone(), torch.empty_like(x)

    kc, vc, out = fresh()
    F.forge_decoder_block(desc, x, out, kc, vc, pos0, ws)       # eager (also the one-time kernel set-up)
    torch.cuda.synchronize()
    ref_out, ref_k = out.clone(), kc.clone()

    kc, vc, out = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            F.forge_decoder_block(desc, x, out, kc, vc, pos0, ws)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        kc.copy_(kc0); vc.copy_(vc0); out.fill_(0)          # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out) and torch.equal(kc, ref_k)
