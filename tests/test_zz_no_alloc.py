"""pt_decode_step_static (the decode step whose temporaries live in the library's static device array, for
callers that cannot allocate) against pt_decode_step, through the C ABI: two calls in a row, the second on a
smaller input, so that whatever the first call left in the array would show."""
import numpy as np
import pytest

from paper_2602_07306_amd import inputs as I
from tests.helpers import small_bf16_config

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _pair(cfg, seed):
    from paper_2602_07306_amd import binding as PB
    a, b = PB.PTModel(cfg), PB.PTModel(cfg)
    a.pt_init_weights(seed)
    b.pt_init_weights(seed)
    return a, b


def _steps(a, b, tokens, feed, hidden=False):
    """Prefills both handles with the same prompt, then decodes the same tokens: handle a through
    pt_decode_step, handle b through pt_decode_step_static.  Returns the two lists of outputs."""
    from paper_2602_07306_amd import binding as PB
    outs = ([], [])
    for m in (a, b):
        m.pt_reset()
        m.pt_prefill(torch.from_numpy(tokens).cuda(), logits_mode=PB.PT_LOGITS_NONE)
    for t in feed:
        dev = torch.from_numpy(np.ascontiguousarray(t)).cuda()
        for k, m in enumerate((a, b)):
            lg, hid, am = m.pt_decode_step(dev, want_hidden=True, want_argmax=True, static_scratch=(k == 1))
            torch.cuda.synchronize()
            outs[k].append((lg.cpu().numpy(), hid.cpu().numpy(), am.cpu().numpy()))
    return outs


def test_static_scratch_decode_equals_the_workspace_decode_twice_in_a_row():
    from paper_2602_07306_amd import binding as PB
    # d = 512: the decode GEMMs run the weight-streaming kernel with K slices left in scratch; one sequence with
    # a 700-token prompt: decode attention splits the keys, so its partials go through scratch as well
    cfg = small_bf16_config(n_tracks=3, n_layers=4, block_depth=2, d_model=512, n_heads=8, n_kv_heads=2, head_dim=64,
                            d_ffn=1536, max_batch=6, max_seq=768, merge_scale=1.0 / 3)
    a, b = _pair(cfg, 41)
    big = I.make_tokens(41, 6, 96, cfg.vocab)
    feed = I.make_tokens(42, 3, 6, cfg.vocab)
    ref, got = _steps(a, b, big, feed)
    for r, g in zip(ref, got):
        for x, y in zip(r, g):
            assert np.array_equal(x, y)
    # second call sequence: a smaller input (one sequence, longer prompt: the split-K attention path)
    small = I.make_tokens(43, 1, 700, cfg.vocab)
    feed = I.make_tokens(44, 3, 1, cfg.vocab)
    b.pt_profile_reset()
    ref, got = _steps(a, b, small, feed)
    for r, g in zip(ref, got):
        for x, y in zip(r, g):
            assert np.array_equal(x, y)
    assert b.pt_profile_paths("attn_decode")[1] == cfg.n_layers * 3      # the tuned kernels ran on the static path
    assert a.pt_seq_len() == b.pt_seq_len() == 703
    a.close()
    b.close()


def test_static_scratch_decode_rejects_a_step_that_does_not_fit():
    from paper_2602_07306_amd import binding as PB
    # 8 tracks x 256 rows x FFN 8192 in bf16 is 32 MiB for the SwiGLU product alone
    cfg = small_bf16_config(n_tracks=8, n_layers=1, block_depth=1, d_model=512, n_heads=8, n_kv_heads=8, head_dim=64,
                            d_ffn=8192, max_batch=256, max_seq=8)
    m = PB.PTModel(cfg)
    m.pt_init_weights(5)
    m.pt_prefill(torch.from_numpy(I.make_tokens(5, 256, 4, cfg.vocab)).cuda(), logits_mode=PB.PT_LOGITS_NONE)
    tok = torch.from_numpy(I.make_tokens(6, 1, 256, cfg.vocab)[0]).cuda()
    with pytest.raises(PB.PTError) as e:
        m.pt_decode_step(tok, static_scratch=True)
    assert e.value.code == PB.PT_ERR_CAPACITY and "static scratch" in str(e.value)
    assert m.pt_seq_len() == 4                      # nothing was launched, the state did not move
    lg, _, _ = m.pt_decode_step(tok)                # the workspace entry point still serves the step
    torch.cuda.synchronize()
    assert np.isfinite(lg.cpu().numpy()).all()
    m.close()
