"""GPU test of the microbatch pipeline (Sec. 2.2): the same batch run as microbatches on separate
streams, eagerly and from one captured graph, must give the single-batch output bit for bit, under
a failure map and across a map change between replays."""
import numpy as np
import pytest
import torch

import synth
from oracle import revive_oracle as orc
from harness import GpuLayer, TOL, f64, rel_err
from synth.resident import MicrobatchPipeline

pytestmark = pytest.mark.gpu

# C4's placement (experts with up to three replicas, five experts lost under its failed ranks)
CFG = synth.scaled(synth.get_config("c4"), T=1200, H=512, I=256, I_shared=256)


@pytest.mark.parametrize("n_micro", [2, 3])
def test_microbatches_match_the_single_batch(n_micro):
    cfg = CFG
    g = GpuLayer(cfg)
    pipe = MicrobatchPipeline(g, n_micro)
    try:
        r = g.forward()
        single = r["out"].clone()
        tr = orc.layer_staged(f64(g.x), None, {e: g.expert_f64(e) for e in range(cfg.E)}, g.shared_f64(), g.p2l,
                              g.oracle_map(), cfg.k, cfg.score_fn, cfg.n_group, cfg.topk_group, logits=f64(r["logits"]))
        assert rel_err(f64(single), tr.out) < TOL[cfg.dtype]

        g.buf["out"].zero_()
        torch.cuda.synchronize()
        pipe.forward()
        torch.cuda.synchronize()
        assert torch.equal(g.buf["out"], single)
        # every microbatch routes like the same tokens of the single batch, replicas included: the oracle's
        # rule on the whole batch, t mod count with t the token's index in the batch
        Tm = cfg.T // n_micro
        for m, (_L, b, _s, _e) in enumerate(pipe.parts):
            assert torch.equal(b["topk_logical"], r["topk_logical"][m * Tm:(m + 1) * Tm])
            assert np.array_equal(b["topk_phys"].cpu().numpy(), tr.topk_phys[m * Tm:(m + 1) * Tm])
            assert np.array_equal(b["topk_weight"].cpu().numpy(), r["topk_weight"][m * Tm:(m + 1) * Tm].cpu().numpy())

        # one graph for all microbatches, replayed across a map change
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            pipe.capture(stream)
            for failed in (cfg.failed_ranks, [], cfg.failed_ranks[:1], cfg.failed_ranks):
                pipe.set_failed(failed, stream=stream)
                g.buf["out"].zero_()
                pipe.replay(stream)
                stream.synchronize()
                got = g.buf["out"].clone()
                want = g.forward(stream=stream)["out"]
                stream.synchronize()
                assert torch.equal(got, want), f"failed ranks {list(failed)}"
    finally:
        pipe.close()
        g.close()
