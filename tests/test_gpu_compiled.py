"""GPU tests of the compiled executor (Sec. "Code Generation: CompiledNPUExecutor"): its
replays must equal the plain launch list bit for bit (same kernels in the same order on the same
data, only the buffer places differ), and the plain launch list is what the oracle gates; the
token model is also checked against the oracle directly."""
import numpy as np
import pytest
import torch

from oracle import forge_oracle as O
from paper_2604_16498_amd import inputs as I
from util import check, check_drift, dev, dev_dict, host

pytestmark = pytest.mark.gpu

SMALL_GPT = I.BlockShape(256, 4, 4, 64, 1024)
SMALL_LLAMA = I.BlockShape(512, 4, 2, 128, 704, norm="rmsnorm", mlp_act="swiglu", use_rope=True,
                           rope_base=500000.0, has_bias=False)


@pytest.fixture(scope="module")
def F():
    from paper_2604_16498_amd import binding
    binding.lib()
    return binding


def replay_and_compare(F, cm, side, out, kc, vc, ref_out, ref_k, ref_v, n=3):
    for _ in range(n):
        out.fill_(0); kc.copy_(ref_k * 0); vc.copy_(ref_v * 0)      # eager work between replays
        torch.cuda.synchronize()
        cm.run(side)
        side.synchronize()
        assert torch.equal(out, ref_out)
        assert torch.equal(kc, ref_k) and torch.equal(vc, ref_v)


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
def test_compiled_token_model_prefill(F, bf16):
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
    model = F.make_model_desc([F.make_block_desc(sh, w) for w in tl], tm)
    tids = torch.from_numpy(ids).cuda()

    # the plain launch list
    plain = torch.zeros(B, S, V, dtype=dt, device="cuda")
    kc0 = torch.zeros(L, B, sh.kv_heads, S, sh.head_dim, dtype=dt, device="cuda"); vc0 = torch.zeros_like(kc0)
    ws0 = F.workspace(F.forge_model_workspace_bytes(model, B, S, S))
    F.forge_model_forward(model, tids, plain, kc0, vc0, 0, ws0)
    torch.cuda.synchronize()

    cm = F.CompiledModel(model, B, S, 0, S)
    ni, nr, _, nb = cm.counts()
    print("compiled: %d instructions, %d registers in %d buffers (rho_buf %.2f), workspace %d B (plain %d B)"
          % (ni, nr, nb, 1 - nb / nr, cm.workspace_bytes(), ws0.numel()))
    out = torch.zeros_like(plain)
    kc = torch.zeros_like(kc0); vc = torch.zeros_like(vc0)
    ws = F.workspace(cm.workspace_bytes())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    cm.bind(tids, out, kc, vc, ws, side)
    side.synchronize()
    assert torch.equal(out, plain) and torch.equal(kc, kc0) and torch.equal(vc, vc0)   # bind's own pass
    replay_and_compare(F, cm, side, out, kc, vc, plain, kc0, vc0)
    if bf16:
        check_drift(out, ref, "compiled model logits")
    else:
        check(out, ref, False, "compiled model logits")
    cm.close()


@pytest.mark.parametrize("decode", [False, True], ids=["prefill", "decode"])
def test_compiled_hidden_state_llama(F, decode):
    """RoPE, grouped heads, SwiGLU; the decode case takes the projections whose reduce step
    carries RoPE and the second norm, and the split-KV attention with its scratch area."""
    sh = SMALL_LLAMA
    L = 3
    B, S, cap, pos0 = (8, 1, 200, 150) if decode else (1, 130, 130, 0)
    wl = I.scaled(I.WORKLOADS[4], block=sh, layers=L, batch=B, seq=S)
    mw = I.model_weights(wl, random_affine=True)
    layers = [I.block_weights(sh, 73, l, bf16=True, random_affine=True) for l in range(L)]
    tl = [dev_dict(w, True) for w in layers]
    tm = dev_dict(mw, True)
    model = F.make_model_desc([F.make_block_desc(sh, w) for w in tl], tm)
    x = dev(I.normal(73, 0, "x", (B, S, sh.d_model), 1.0, bf16=True), True)
    k_init = dev(I.normal(73, 0, "k_cache", (L, B, sh.kv_heads, cap, sh.head_dim), 1.0, bf16=True), True)
    v_init = dev(I.normal(73, 0, "v_cache", (L, B, sh.kv_heads, cap, sh.head_dim), 1.0, bf16=True), True)

    plain = torch.empty(B, S, sh.d_model, dtype=torch.bfloat16, device="cuda")
    kc0, vc0 = k_init.clone(), v_init.clone()
    ws0 = F.workspace(F.forge_model_workspace_bytes(model, B, S, cap))
    F.forge_model_forward(model, x, plain, kc0, vc0, pos0, ws0)
    torch.cuda.synchronize()

    cm = F.CompiledModel(model, B, S, pos0, cap)
    out = torch.zeros_like(plain)
    kc, vc = k_init.clone(), v_init.clone()
    ws = F.workspace(cm.workspace_bytes())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    cm.bind(x, out, kc, vc, ws, side)
    side.synchronize()
    assert torch.equal(out, plain) and torch.equal(kc, kc0) and torch.equal(vc, vc0)
    for _ in range(3):
        out.fill_(0); kc.copy_(k_init); vc.copy_(v_init)
        torch.cuda.synchronize()
        cm.run(side)
        side.synchronize()
        assert torch.equal(out, plain) and torch.equal(kc, kc0) and torch.equal(vc, vc0)

    # bind again to other tensors: the new graph writes there and leaves the old ones alone
    out2 = torch.zeros_like(plain)
    kc2, vc2 = k_init.clone(), v_init.clone()
    out.fill_(0)
    torch.cuda.synchronize()
    cm.bind(x, out2, kc2, vc2, ws, side)
    cm.run(side)
    side.synchronize()
    assert torch.equal(out2, plain) and torch.equal(kc2, kc0)
    assert torch.all(out == 0)
    cm.close()


def test_compiled_bind_rejects_small_workspace_and_run_before_bind(F):
    sh = SMALL_GPT
    w = dev_dict(I.block_weights(sh, 71, 0, bf16=True), True)
    wl = I.scaled(I.WORKLOADS[4], block=sh, layers=1, batch=1, seq=64)
    tm = dev_dict(I.model_weights(wl), True)
    model = F.make_model_desc([F.make_block_desc(sh, w)], tm)
    cm = F.CompiledModel(model, 1, 64, 0, 64)
    x = torch.zeros(1, 64, sh.d_model, dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(x)
    kc = torch.zeros(1, 1, sh.kv_heads, 64, sh.head_dim, dtype=torch.bfloat16, device="cuda"); vc = torch.zeros_like(kc)
    side = torch.cuda.Stream()
    with pytest.raises(F.ForgeError) as e:
        cm.bind(x, out, kc, vc, F.workspace(256), side)
    assert e.value.status == 3
    with pytest.raises(F.ForgeError) as e:
        cm.run(side)
    assert e.value.status == 1
    cm.close()
