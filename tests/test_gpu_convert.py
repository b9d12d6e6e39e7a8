"""meld_linears + MeldedOptimizer on a small, randomly initialised LLaMA-style model (no download)."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def _tiny_llama():
    transformers = pytest.importorskip("transformers")
    cfg = transformers.LlamaConfig(vocab_size=512, hidden_size=256, intermediate_size=512, num_hidden_layers=2,
                                   num_attention_heads=4, num_key_value_heads=4, max_position_embeddings=128)
    torch.manual_seed(0)
    return transformers.LlamaForCausalLM(cfg).to(device="cuda", dtype=torch.bfloat16)


def test_melded_model_matches_the_original_closely_and_learns():
    from paper_2510_24061_amd.convert import MeldedOptimizer, meld_linears
    from paper_2510_24061_amd.nn import MeldedLoRALinear
    model = _tiny_llama()
    for p in model.parameters():
        p.requires_grad_(False)
    ids = torch.randint(0, 512, (4, 64), generator=torch.Generator().manual_seed(1)).cuda()
    with torch.no_grad():
        loss_before = float(model(input_ids=ids, labels=ids).loss)
    layers = meld_linears(model, rank=16, top_k=lambda m: m // 4)
    assert len(layers) == 14 and all(isinstance(l, MeldedLoRALinear) for l in layers)
    assert isinstance(model.model.layers[1].mlp.down_proj, MeldedLoRALinear)
    assert isinstance(model.lm_head, torch.nn.Linear)                          # not in the list: untouched
    # FP8 backbone + adapter in place of bf16 weights: the loss of the untrained model barely moves
    with torch.no_grad():
        assert float(model(input_ids=ids, labels=ids).loss) == pytest.approx(loss_before, abs=0.1)
    opt = MeldedOptimizer(layers, lr=3e-3, max_norm=1.0)
    wq0 = [l.wq.clone() for l in layers]
    losses = []
    for _ in range(40):
        # called the ordinary way: the embedding and the norms are frozen, so the first block's q, k and v
        # projections see an input without a gradient and must still form theirs
        loss = model(input_ids=ids, labels=ids).loss
        loss.backward()
        assert all(l.backward_calls == 1 for l in layers)
        opt.step()
        losses.append(float(loss.detach()))
    print("loss every 5 steps:", [round(v, 3) for v in losses[::5]], flush=True)
    assert all(map(lambda v: v == v and v < 1e4, losses))
    assert losses[-1] < losses[0] - 0.3, losses[::5]                            # memorising four sequences
    m_rows = [l.out_features for l in layers]
    for l, w0, m in zip(layers, wq0, m_rows):
        assert not torch.equal(l.wq[:m], w0[:m])                               # rows were folded
        assert torch.equal(l.wq[m:], w0[m:])                                   # the adapter rows never change


def test_bias_is_kept_and_odd_sizes_are_refused():
    from paper_2510_24061_amd.convert import meld_linears
    net = torch.nn.Sequential()
    net.add_module("up_proj", torch.nn.Linear(64, 48, bias=True))
    net = net.cuda()
    x = torch.randn(32, 64, device="cuda")
    want = net(x)
    layers = meld_linears(net, rank=16, top_k=8)
    got = net(x.to(torch.bfloat16)).float()
    assert len(layers) == 1
    assert torch.linalg.norm(got - want) / torch.linalg.norm(want) < 0.08      # FP8 activations and weights
    bad = torch.nn.Sequential()
    bad.add_module("up_proj", torch.nn.Linear(40, 48))
    with pytest.raises(ValueError):
        meld_linears(bad.cuda(), rank=16, top_k=8)
