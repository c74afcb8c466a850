"""GPU parity of the decode step with per-sequence lengths (the generation loop of the paper's
language-modelling workload, Sec. "Datasets": a prompt, then one token at a time) against the
fp64 oracle.  The oracle has no notion of a ragged batch: every sequence is checked on its own
against the oracle run with that sequence's length."""
import math

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


def tdtype(bf16):
    return torch.bfloat16 if bf16 else torch.float32


def ipos(pos):
    return torch.tensor(pos, dtype=torch.int32, device="cuda")


@pytest.mark.parametrize("bf16,Hq,Hkv,dh", [(True, 8, 2, 128), (True, 4, 4, 64), (True, 8, 1, 64), (False, 4, 2, 64)],
                         ids=["g4_d128", "g1_d64", "g8_d64_valu", "f32"])
def test_attn_decode_varlen(F, bf16, Hq, Hkv, dh):
    pos = [0, 3, 255, 256, 700, 511, 1]              # lengths 1 .. 701: some sequences end before the later KV splits begin
    B, cap = len(pos), 704
    q = I.normal(96, 0, "q", (B, Hq, 1, dh), 1.0, bf16=bf16)
    k = I.normal(96, 0, "k_cache", (B, Hkv, cap, dh), 1.0, bf16=bf16)
    v = I.normal(96, 0, "v_cache", (B, Hkv, cap, dh), 1.0, bf16=bf16)
    scale = 1.0 / math.sqrt(dh)
    out = torch.empty(B, 1, Hq * dh, dtype=tdtype(bf16), device="cuda")
    max_pos = max(pos)
    ws = F.workspace(F.forge_attn_fused_workspace_bytes(B, Hq, Hkv, 1, max_pos + 1, dh, tdtype(bf16)))
    F.forge_attn_decode_varlen(dev(q, bf16), dev(k, bf16), dev(v, bf16), out, ipos(pos), max_pos, scale, ws)
    torch.cuda.synchronize()
    for b, p in enumerate(pos):
        ref = O.attention(q[b:b + 1], k[b:b + 1, :, :p + 1], v[b:b + 1, :, :p + 1], scale, True)
        check(out[b:b + 1], ref, bf16, "sequence %d (length %d)" % (b, p + 1))


def test_attn_decode_varlen_clamps_bad_positions(F):
    """Entries outside [0, max_pos] are clamped on the device: such a sequence gets the result
    for the clamped length, and nothing outside the cache is touched."""
    B, Hq, Hkv, dh, cap, max_pos = 3, 4, 2, 64, 64, 40
    q = I.normal(97, 0, "q", (B, Hq, 1, dh), 1.0, bf16=True)
    k = I.normal(97, 0, "k_cache", (B, Hkv, cap, dh), 1.0, bf16=True)
    v = I.normal(97, 0, "v_cache", (B, Hkv, cap, dh), 1.0, bf16=True)
    out = torch.empty(B, 1, Hq * dh, dtype=torch.bfloat16, device="cuda")
    ws = F.workspace(F.forge_attn_fused_workspace_bytes(B, Hq, Hkv, 1, max_pos + 1, dh, torch.bfloat16))
    F.forge_attn_decode_varlen(dev(q, True), dev(k, True), dev(v, True), out, ipos([-5, 1000000, 7]), max_pos, None, ws)
    torch.cuda.synchronize()
    for b, p in enumerate([0, max_pos, 7]):
        ref = O.attention(q[b:b + 1], k[b:b + 1, :, :p + 1], v[b:b + 1, :, :p + 1], 1.0 / math.sqrt(dh), True)
        check(out[b:b + 1], ref, True, "clamped sequence %d" % b)


GPT = I.BlockShape(256, 4, 4, 64, 1024)
LLAMA = I.BlockShape(512, 8, 2, 64, 768, norm="rmsnorm", mlp_act="swiglu", use_rope=True,
                     rope_base=500000.0, has_bias=False)


@pytest.mark.parametrize("sh,bf16,B", [(LLAMA, True, 6), (GPT, True, 5), (GPT, False, 4), (LLAMA, True, 70)],
                         ids=["llama_bf16", "gpt_bf16", "gpt_f32", "llama_bf16_70_sequences"])
def test_block_decode_varlen(F, sh, bf16, B):
    """One decoder layer, one new token per sequence, every sequence at its own position.  Up to
    64 bf16 sequences take the projections whose reduce step carries RoPE and the second norm;
    fp32 and 70 sequences take the tile kernels and the separate RoPE launches."""
    cap = 300
    rng = np.random.default_rng(98)
    pos = [int(p) for p in rng.integers(0, cap - 1, size=B)]
    pos[0], pos[1] = 0, cap - 1
    w = I.block_weights(sh, 98, 0, bf16=bf16, random_affine=True, weight_std=0.05)
    x = I.normal(98, 0, "x", (B, 1, sh.d_model), 1.0, bf16=bf16)
    kc = I.normal(98, 0, "k_cache", (B, sh.kv_heads, cap, sh.head_dim), 1.0, bf16=bf16)
    vc = I.normal(98, 0, "v_cache", (B, sh.kv_heads, cap, sh.head_dim), 1.0, bf16=bf16)
    tw = dev_dict(w, bf16)                       # the descriptor holds raw pointers: keep the tensors
    desc = F.make_block_desc(sh, tw)
    tx, tk, tv = dev(x, bf16), dev(kc, bf16), dev(vc, bf16)
    out = torch.empty_like(tx)
    ws = F.workspace(F.forge_decoder_block_workspace_bytes(desc, B, 1, cap))
    F.forge_decoder_block_decode(desc, tx, out, tk, tv, ipos(pos), max(pos), ws)
    torch.cuda.synchronize()
    gk, gv = host(tk), host(tv)
    for b, p in enumerate(pos):
        kr, vr = kc[b:b + 1].astype(np.float64), vc[b:b + 1].astype(np.float64)
        ref = O.decoder_block(sh, w, x[b:b + 1], kr, vr, pos0=p)
        check(out[b:b + 1], ref, bf16, "sequence %d at position %d" % (b, p), chain=True)
        check(tk[b:b + 1, :, p], kr[:, :, p], bf16, "new k row of sequence %d" % b)
        check(tv[b:b + 1, :, p], vr[:, :, p], bf16, "new v row of sequence %d" % b)
        # every other cache row of the sequence is untouched
        keep = np.ones(cap, dtype=bool); keep[p] = False
        assert np.array_equal(gk[b][:, keep], kc[b][:, keep].astype(np.float64))
        assert np.array_equal(gv[b][:, keep], vc[b][:, keep].astype(np.float64))


@pytest.mark.parametrize("padded", [False, True], ids=["prompts_one_by_one", "prompts_in_one_launch"])
@pytest.mark.parametrize("compiled", [False, True], ids=["plain", "compiled"])
def test_generation_loop_ragged_batch(F, compiled, padded):
    """Three prompts of different lengths, then 6 tokens each (teacher-forced ids): the logits of
    step i of sequence b equal row len_b + i of one causal forward of that sequence, which is
    what the oracle computes.  The compiled variant records the decode step ONCE and replays it
    for every step while the positions advance in device memory.

    prompts_in_one_launch: the prompts go through ONE prefill launch, padded on the right to the
    longest with token 0.  Under the causal mask a query at position i < len_b sees keys 0..i only,
    so the rows of a sequence's own prompt come out as if it had run alone; the rows past len_b
    (logits and cache) hold the padding's values, which the decode steps never read: step i writes
    cache row len_b + i before it attends rows 0..len_b + i."""
    sh = GPT
    L, V, cap, steps = 2, 520, 64, 6
    lens = [5, 17, 24]
    B = len(lens)
    wl = I.scaled(I.WORKLOADS[2], block=sh, layers=L, vocab=V, n_pos=64, batch=B, seq=max(lens) + steps, bf16=True)
    mw = I.model_weights(wl, random_affine=True)
    layers = [I.block_weights(sh, 99, l, bf16=True, random_affine=True) for l in range(L)]
    ids = I.token_ids(99, B, max(lens) + steps, V)
    refs = [O.gpt_forward(sh, layers, mw, ids=ids[b:b + 1, :lens[b] + steps]) for b in range(B)]
    tl = [dev_dict(w, True) for w in layers]
    tm = dev_dict(mw, True)
    model = F.make_model_desc([F.make_block_desc(sh, w) for w in tl], tm)
    tids = torch.from_numpy(ids).cuda()
    kc = torch.zeros(L, B, sh.kv_heads, cap, sh.head_dim, dtype=torch.bfloat16, device="cuda"); vc = torch.zeros_like(kc)

    if padded:
        n = max(lens)
        pids = torch.zeros(B, n, dtype=tids.dtype, device="cuda")
        for b in range(B):
            pids[b, :lens[b]] = tids[b, :lens[b]]
        lg = torch.empty(B, n, V, dtype=torch.bfloat16, device="cuda")
        ws = F.workspace(F.forge_model_workspace_bytes(model, B, n, cap))
        F.forge_model_forward(model, pids, lg, kc, vc, 0, ws)
        torch.cuda.synchronize()
        for b in range(B):
            check_drift(lg[b:b + 1, :lens[b]], refs[b][:, :lens[b]], "prompt of sequence %d (padded batch)" % b)
    # prompts: one sequence at a time into a cache of its own, copied into the batched cache
    for b, n in enumerate([] if padded else lens):
        k1 = torch.zeros(L, 1, sh.kv_heads, cap, sh.head_dim, dtype=torch.bfloat16, device="cuda"); v1 = torch.zeros_like(k1)
        lg = torch.empty(1, n, V, dtype=torch.bfloat16, device="cuda")
        ws = F.workspace(F.forge_model_workspace_bytes(model, 1, n, cap))
        F.forge_model_forward(model, tids[b:b + 1, :n].contiguous(), lg, k1, v1, 0, ws)
        torch.cuda.synchronize()
        check_drift(lg, refs[b][:, :n], "prompt of sequence %d" % b)
        kc[:, b] = k1[:, 0]; vc[:, b] = v1[:, 0]

    seq_pos = ipos(lens)
    max_pos = max(lens) + steps - 1
    tok = torch.empty(B, 1, dtype=torch.int32, device="cuda")
    logits = torch.empty(B, 1, V, dtype=torch.bfloat16, device="cuda")
    side = torch.cuda.Stream()
    if compiled:
        cm = F.CompiledModel(model, B, 1, max_pos, cap)
        ws = F.workspace(cm.workspace_bytes())
        for b in range(B):
            tok[b, 0] = tids[b, lens[b]]
        torch.cuda.synchronize()
        k_keep, v_keep = kc.clone(), vc.clone()
        cm.bind_decode(tok, logits, kc, vc, seq_pos, ws, side)      # runs step 0 once while binding
        side.synchronize()
        kc.copy_(k_keep); vc.copy_(v_keep)                          # start the loop from the prompts again
    else:
        ws = F.workspace(F.forge_model_workspace_bytes(model, B, 1, cap))
    worst = 0.0
    for i in range(steps):
        for b in range(B):
            tok[b, 0] = tids[b, lens[b] + i]
        torch.cuda.synchronize()
        if compiled:
            cm.run(side)
            side.synchronize()
        else:
            F.forge_model_decode(model, tok, logits, kc, vc, seq_pos, max_pos, ws)
            torch.cuda.synchronize()
        got = host(logits)
        for b in range(B):
            _, l2 = check_drift(got[b], refs[b][0, lens[b] + i:lens[b] + i + 1], "step %d sequence %d" % (i, b))
            worst = max(worst, l2)
        seq_pos += 1                                                # the positions advance on the device
    print("ragged generation loop (%s): worst l2 %.3e" % ("compiled" if compiled else "plain", worst))
    if compiled:
        cm.close()


def test_decode_varlen_rejects(F):
    sh = GPT
    tw = dev_dict(I.block_weights(sh, 95, 0, bf16=True), True)
    desc = F.make_block_desc(sh, tw)
    x = torch.zeros(2, 1, sh.d_model, dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros(2, sh.kv_heads, 16, sh.head_dim, dtype=torch.bfloat16, device="cuda")
    ws = F.workspace(F.forge_decoder_block_workspace_bytes(desc, 2, 1, 16))
    with pytest.raises(F.ForgeError) as e:           # max_pos must lie inside the cache
        F.forge_decoder_block_decode(desc, x, torch.empty_like(x), kc, kc.clone(), ipos([1, 2]), 16, ws)
    assert e.value.status == 1
