"""The seeded input generators: one value per (seed, index) whatever the route."""
import numpy as np
import torch

from workloads import configs, prng


def test_three_routes_to_the_same_bits():
    n = 5000
    a = prng.randn_bf16(77, n).view(torch.int16).numpy().astype(np.uint16)
    b = prng.randn_bf16_np(77, n)
    assert (a == b).all()
    tab = prng.normal_table_u16()
    for i in (0, 1, 4999):
        assert b[i] == tab[prng.splitmix64_scalar(77, i) >> 48]
    # chunking does not change values
    c = prng.randn_bf16(77, n, chunk=1024).view(torch.int16).numpy().astype(np.uint16)
    assert (a == c).all()


def test_values_look_standard_normal():
    x = prng.randn_bf16(prng.sub_seed(1, 2), 1 << 18).float()
    assert abs(x.mean().item()) < 0.01 and abs(x.std().item() - 1.0) < 0.01
    assert torch.isfinite(x).all() and x.abs().max() < 5.0


def test_config1_lengths_follow_the_recipe():
    for step in range(16):
        lens = configs.tiny_lengths(step)
        assert len(lens) == 4 and (lens >= 1).all() and (lens <= 17).all() and lens.sum() <= 64
    wl = configs.config1_tiny()
    calls = wl.step_calls(3)
    assert len(calls) == 8 and calls[0].tensor.shape == (64, 256)
    r = calls[0].reqs
    lens = configs.tiny_lengths(3)
    assert (r[:, 2] == lens - 1).all() and (r[:, 3] == 1).all()
    assert (r[:, 1] == np.concatenate([[0], np.cumsum(lens)[:-1]])).all()


def test_config_shapes_scaled_down():
    w2 = configs.config2_decode8b(n_points=2, n_steps=2)
    c = w2.step_calls(1)[1]
    assert c.tensor.shape == (64, 4096) and c.summary_mask == 5 and c.reqs.shape == (64, 5)
    w3 = configs.config3_prefill(n_reqs=3, len_lo=5, len_hi=40, hidden=64, inter=96, n_resid=2, n_mlp=1)
    calls = w3.step_calls(0)
    assert [c.point_id for c in calls] == [0, 100, 1]
    lens = prng.randint(prng.sub_seed(3, 9, 0), 3, 5, 40)
    assert (calls[0].reqs[:, 3] == -(-lens // 4)).all() and (calls[0].reqs[:, 4] == 4).all()
    assert int(calls[0].reqs[-1, 1] + (calls[0].reqs[-1, 3] - 1) * 4) < calls[0].tensor.shape[0]
    w4 = configs.config4_paged_kv(n_layers_cap=1, n_blocks=512, n_reqs=6, ctx_lo=10, ctx_hi=200,
                                  reqs_per_step=2, n_steps=3)
    calls = w4.step_calls(2)
    assert len(calls) == 2 and calls[0].paged.block_table.shape == (6, 13)
    bt = calls[0].paged.block_table.numpy()
    ctx0 = w4.notes["ctx0"]
    used = np.concatenate([bt[r, : -(-(ctx0[r] + 3) // 16)] for r in range(6)])
    assert len(set(used.tolist())) == len(used)          # physical blocks are not shared
    assert (calls[0].reqs[:, 3] == ctx0[calls[0].reqs[:, 1]] + 2).all()
