"""Parity at the benchmark's full size and launch configuration: the Large PT prefill of bench.py (8 tracks x 32
layers, batch 8 x 4096 tokens, seed 3) runs on the GPU exactly as it is timed; the oracle then computes sampled
outputs one by one.  Causality makes that affordable: positions 0 .. P-1 of a sequence depend on its first P tokens
only (pinned for the oracle by the causal-prefix test), so the oracle runs the P-token prefix of one of the eight
sequences, with the model's weights generated layer by layer (they do not fit the host at once).

By default the oracle follows the first track block (8 layers of all 8 tracks and the merge after it: the first
block tap of the full-depth GPU run).  PT_LONG_TESTS=1 follows all 32 layers and compares every tap and the logits
(about five minutes of host time, nearly all of it weight generation)."""
import dataclasses
import os
import sys

import numpy as np
import pytest

from oracle import pt_oracle as O
from paper_2602_07306_amd import inputs as I
from tests.helpers import BF16_TOL, assert_close, path_counts

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def test_large_prefill_at_full_size_matches_the_oracle_on_sampled_positions(capsys):
    from paper_2602_07306_amd import binding as PB
    full = os.environ.get("PT_LONG_TESTS") == "1"
    B, S, P, picks = 8, 4096, 64, (5,)
    cfg = I.config_large(max_batch=B, max_seq=S)
    tokens = I.make_tokens(3, B, S, cfg.vocab)
    model = PB.PTModel(cfg)
    model.pt_init_weights(3)
    model.pt_profile_reset()
    taps, _ = model.pt_set_taps(B * S)
    logits, _ = model.pt_prefill(torch.from_numpy(tokens).cuda(), logits_mode=PB.PT_LOGITS_ALL)
    torch.cuda.synchronize()
    model.pt_sync_status()
    assert model.pt_merge_count() == cfg.n_merges
    counts = path_counts(model)      # the launch configuration bench.py times: tuned kernels everywhere
    for c in ("gemm_qkv", "gemm_out", "gemm_gateup", "gemm_down"):
        assert counts[c] == [0, cfg.n_layers, 0, 0], (c, counts[c])
    assert counts["attn_prefill"] == [0, cfg.n_layers, 0, 0]
    got_taps = [taps[k].view(B, S, -1)[list(picks), :P].cpu().numpy() for k in range(cfg.n_merges)]
    got_logits = logits.view(B, S, -1)[list(picks), :P].cpu().numpy()
    model.close()
    del taps, logits
    torch.cuda.empty_cache()

    ocfg = cfg if full else dataclasses.replace(cfg, n_layers=cfg.block_depth)

    def progress(name, track, layer):   # one line per layer, past pytest's capture: the oracle works for minutes
        if name == "wq" and track == 0:
            with capsys.disabled():
                print("oracle: layer %d of %d" % (layer + 1, ocfg.n_layers), file=sys.stderr, flush=True)

    W = I.LazyWeights(ocfg, 3, on_tensor=progress)
    for j, b in enumerate(picks):
        st = O.PTState(ocfg, 1, P)
        ref = O.pt_prefill(ocfg, W, st, tokens=tokens[b:b + 1, :P], collect_taps=True)
        for k in range(ocfg.n_merges):
            assert_close(got_taps[k][j], ref["taps"][0][k], BF16_TOL, "tap %d of sequence %d" % (k, b))
        if full:
            assert_close(got_logits[j], ref["logits"][0], BF16_TOL, "logits of sequence %d" % b)
