"""The shared seeded input generator: determinism, addressability, distribution."""
import torch

from synthdata import CONFIGS, gen_prompt, gen_tensor, get_config, iter_tensor_specs, tensor_shape
from synthdata.generator import _mix, _mix_int, _s64


def test_mix_matches_python_integers():
    vals = [0, 1, 0xDEADBEEF, (1 << 63) + 12345, (1 << 64) - 1]
    t = _mix(torch.tensor([_s64(v) for v in vals]))
    assert [x & ((1 << 64) - 1) for x in t.tolist()] == [_mix_int(v) for v in vals]


def test_chunking_does_not_change_values():
    cfg = get_config("mini_gqa")
    a = gen_tensor(cfg, 2, "wd", chunk=1000)
    b = gen_tensor(cfg, 2, "wd", chunk=1 << 20)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_distribution_and_branch_scaling():
    cfg = get_config("tiny")
    w0 = gen_tensor(cfg, 0, "wd").double()
    w2 = gen_tensor(cfg, 2, "wd").double()
    assert abs(w0.mean().item()) < 2e-4
    assert abs(w0.std().item() / 0.02 - 1) < 0.02
    assert abs(w2.std().item() / (0.02 * 0.25) - 1) < 0.02
    assert not torch.equal(gen_tensor(cfg, 0, "wq"), gen_tensor(cfg, 0, "wk"))
    assert not torch.equal(gen_tensor(cfg, 0, "wq"), gen_tensor(cfg, 1, "wq"))
    assert gen_tensor(cfg, 0, "attn_norm").eq(1).all()
    g = gen_tensor(get_config("mini_gqa"), 0, "attn_norm")
    assert g.dtype == torch.float32 and abs(g.mean().item() - 1) < 0.02 and g.std().item() > 0.05


def test_shapes_dtypes_and_tying():
    for cfg in (get_config("tiny"), get_config("mini_gqa")):
        for layer, kind in iter_tensor_specs(cfg):
            if layer > 0:
                continue
            t = gen_tensor(cfg, layer, kind)
            assert tuple(t.shape) == tensor_shape(cfg, kind)
            if not kind.endswith("norm"):
                assert t.dtype == (torch.bfloat16 if cfg.weight_dtype == "bf16" else torch.float32)
    cfg = get_config("mini_gqa")
    assert torch.equal(gen_tensor(cfg, -1, "lm_head").view(torch.int16),
                       gen_tensor(cfg, -1, "embed").view(torch.int16))


def test_prompt_range_and_prefix_property():
    for name, cfg in CONFIGS.items():
        p = gen_prompt(cfg, length=min(cfg.prompt_len, 64))
        assert p.dtype == torch.int32 and int(p.min()) >= 0 and int(p.max()) < cfg.vocab
    cfg = get_config("tiny")
    assert torch.equal(gen_prompt(cfg, length=10), gen_prompt(cfg)[:10])


def test_config_table_matches_stated_shapes():
    c = get_config("llama7b")
    assert (c.n_layers, c.d_model, c.n_q_heads, c.n_kv_heads, c.head_dim, c.d_ffn, c.vocab) == \
        (32, 4096, 32, 32, 128, 11008, 32000)
    assert c.layer_weight_bytes() == 404750336 and c.head_weight_bytes() == 262144000
    c = get_config("llama70b")
    assert abs(c.n_params() * 2 / 1e9 - 137.95) < 0.1
    for c in CONFIGS.values():
        assert c.n_q_heads % c.n_kv_heads == 0 and c.head_dim % 16 == 0 and c.d_ffn % 8 == 0
