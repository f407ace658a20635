"""wind_beam_window_scores_static, the entry point that allocates nothing and does not wait: called
through the C ABI on two shapes in a row, the second smaller than the first (the static scratch
array then still holds the first call's rows), and checked against wind_beam_window_scores on the
same inputs.  Both run the same kernels, so labels, jumps and scores must agree bit for bit.  Shapes
whose scratch layout does not fit the static array are refused with a message."""
import numpy as np
import pytest

import wind_inputs as wi

pytestmark = pytest.mark.gpu


def random_inputs(torch, cfg, n, Bh, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    enc = torch.randn((n, cfg.D), generator=g, dtype=torch.float32).cuda()
    dec = (0.5 * torch.randn((Bh, cfg.Hp), generator=g, dtype=torch.float32)).cuda()
    return enc, dec


@pytest.mark.parametrize("name,shapes,exact", [("greedy_b1", ((16, 16, 8), (5, 3, 8), (16, 23, 4)), 0),   # few-rows logits kernel, then > 256 rows
                                               ("greedy_b1", ((9, 40, 8), (3, 2, 32)), 1),               # tile kernel with the split hidden vector
                                               ("tiny", ((16, 6, 8), (4, 3, 5)), 0)])                    # fp32 model
def test_static_entry_point_equals_the_allocating_one(name, shapes, exact):
    import torch
    from paper_2505_13765_amd import WindModel

    assert torch.cuda.is_available(), "this test needs the MI355X"
    cfg = wi.CONFIGS[name]
    m = WindModel.from_config(cfg, wi.make_weights(cfg))
    m.set_option("beam_exact", exact)
    for i, (n, Bh, K) in enumerate(shapes):
        enc, dec = random_inputs(torch, cfg, n, Bh, 1000 * i + n)
        ref = m.beam_window_scores(enc, dec, K)
        out = (torch.full((Bh, K), -9, dtype=torch.int32, device="cuda"), torch.full((Bh, K), -9, dtype=torch.int32, device="cuda"),
               torch.full((Bh, K), float("nan"), dtype=torch.float32, device="cuda"))
        m.beam_window_scores_static(enc, dec, K, out)
        torch.cuda.synchronize()
        got = [t.cpu().numpy() for t in out]
        print(f"{name} n={n} Bh={Bh} K={K} exact={exact}: best pairs {got[0][0, :3].tolist()} scores {got[2][0, :3].tolist()}", flush=True)
        assert (got[0] == ref[0]).all() and (got[1] == ref[1]).all()
        assert got[2].tobytes() == ref[2].tobytes()
    m.close()


def test_static_entry_point_refuses_what_does_not_fit():
    import torch
    from paper_2505_13765_amd import WindModel
    from paper_2505_13765_amd.binding import WindError

    cfg = wi.CONFIGS["greedy_b1"]
    m = WindModel.from_config(cfg, wi.make_weights(cfg))
    n, Bh, K = 64, 64, 4                      # 4096 rows x 1025 logits x 4 bytes alone are 16.8 MB
    enc, dec = random_inputs(torch, cfg, n, Bh, 5)
    out = (torch.zeros((Bh, K), dtype=torch.int32, device="cuda"), torch.zeros((Bh, K), dtype=torch.int32, device="cuda"),
           torch.zeros((Bh, K), dtype=torch.float32, device="cuda"))
    with pytest.raises(WindError, match="static buffer"):
        m.beam_window_scores_static(enc, dec, K, out)
    m.beam_window_scores(enc, dec, K)         # the allocating entry point takes the same shape
    m.close()
