"""asynclm_greedy_token_static, the entry point that allocates nothing (its kernel's scratch is a static array in device
memory), against asynclm_peek_token, the existing entry point it is a variant of: both must pick the same token.
Integer work, so the bar is exact equality.  Two calls in a row on one stream, the second over a smaller vocabulary
(the static scratch keeps the first call's partial results), with and without ids to skip, through the C ABI."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import asynclm_inputs as ai

pytestmark = pytest.mark.gpu


def _peek_and_static(pkg, model, banned, stream, prompt_len):
    dev = torch.device("cuda:0")
    w_dev = ai.make_weights(model, device=dev)
    lm = pkg.AsyncLM(model, w_dev, max_positions=64, stream=stream)
    lm.prefill(0, ai.uniform_tokens(ai.MASTER_SEED, 950, prompt_len, model.vocab))
    lm.set_banned_tokens(0, banned)
    want = lm.peek_choice(0)                                   # existing entry point (synchronises)
    logits = lm.logits(0)
    ban_dev = torch.tensor(banned, dtype=torch.int32, device=dev) if banned else None
    out = torch.full((1,), -7, dtype=torch.int32, device=dev)
    rc = pkg.greedy_token_static(lm.logits_device(0), model.vocab, ban_dev.data_ptr() if banned else 0, len(banned),
                                 out.data_ptr(), stream.cuda_stream)
    assert rc == 0
    stream.synchronize()
    got = int(out.item())
    lm.close()
    return want, got, logits


def test_static_greedy_token_equals_peek_token_on_two_calls_the_second_smaller():
    import paper_2412_07017_amd as pkg
    stream = torch.cuda.Stream()
    tiny = ai.preset("tiny").model
    # first call: vocabulary 5000 (three blocks of the kernel), the two best ids skipped
    big = replace(tiny, vocab=5000)
    w0, g0, lg0 = _peek_and_static(pkg, big, [], stream, 9)
    assert w0 == g0 == int(np.argmax(lg0))
    top = [int(v) for v in np.argsort(-lg0)[:2]]
    w1, g1, lg1 = _peek_and_static(pkg, big, top, stream, 9)
    assert w1 == g1 == int(np.argsort(-lg1)[2])
    # second call: a smaller vocabulary (one block, ragged size), right after, on the same stream
    small = replace(tiny, vocab=601)
    w2, g2, lg2 = _peek_and_static(pkg, small, [int(np.argmax(lg0)) % 601], stream, 5)
    assert w2 == g2
    w3, g3, lg3 = _peek_and_static(pkg, small, [], stream, 5)
    assert w3 == g3 == int(np.argmax(lg3))


def test_static_greedy_token_rejects_sizes_beyond_its_limits():
    import paper_2412_07017_amd as pkg
    dev = torch.device("cuda:0")
    x = torch.zeros(16, dtype=torch.float32, device=dev)
    out = torch.zeros(1, dtype=torch.int32, device=dev)
    ban = torch.zeros(64, dtype=torch.int32, device=dev)
    s = torch.cuda.current_stream().cuda_stream
    assert pkg.greedy_token_static(x.data_ptr(), (1 << 24) + 1, 0, 0, out.data_ptr(), s) == pkg.E_INVAL
    assert pkg.greedy_token_static(x.data_ptr(), 0, 0, 0, out.data_ptr(), s) == pkg.E_INVAL
    assert pkg.greedy_token_static(x.data_ptr(), 16, ban.data_ptr(), 32, out.data_ptr(), s) == pkg.E_INVAL
    assert pkg.greedy_token_static(x.data_ptr(), 16, 0, 3, out.data_ptr(), s) == pkg.E_INVAL
    assert pkg.greedy_token_static(0, 16, 0, 0, out.data_ptr(), s) == pkg.E_INVAL
    assert pkg.greedy_token_static(x.data_ptr(), 16, 0, 0, 0, s) == pkg.E_INVAL
    # all-equal logits: the lowest index wins; with it skipped, the next one
    assert pkg.greedy_token_static(x.data_ptr(), 16, 0, 0, out.data_ptr(), s) == 0
    torch.cuda.synchronize()
    assert int(out.item()) == 0
    assert pkg.greedy_token_static(x.data_ptr(), 16, ban.data_ptr(), 1, out.data_ptr(), s) == 0
    torch.cuda.synchronize()
    assert int(out.item()) == 1
