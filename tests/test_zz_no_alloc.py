"""The top-k call that allocates nothing (static scratch inside the library) against the call with caller scratch:
identical tokens and log-probabilities, on two calls in a row, the second with a smaller input (the scratch keeps
the first call's contents), and the size limit is an error."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_static_scratch_topk_equals_caller_scratch_topk():
    import torch
    import paper_2408_15766_amd as P
    assert torch.cuda.is_available()
    rng = np.random.default_rng(123)
    for rows, vocab, k in [(10, 128256, 10), (3, 5000, 16)]:          # second call: fewer rows, fewer slices
        logits = torch.from_numpy((rng.standard_normal((rows, vocab)) * 1.3).astype(np.float32)).cuda()
        want_tok, want_lp = P.spec_k_topk_logprob(logits, k)
        tok = torch.full((rows, 16), -1, dtype=torch.int32, device="cuda")
        lp = torch.full((rows, 16), float("nan"), dtype=torch.float32, device="cuda")
        got_tok, got_lp = P.spec_k_topk_logprob_static(logits, k, tok, lp)
        torch.cuda.synchronize()
        assert torch.equal(got_tok, want_tok)
        assert torch.equal(got_lp, want_lp)                            # same kernels, same order: the same bits
    big = torch.zeros((1, 262144 + 1), dtype=torch.float32, device="cuda")
    with pytest.raises(P.SpecError) as e:
        P.spec_k_topk_logprob_static(big, 4)
    assert e.value.code == P.binding.SPEC_ECAP
    ok_tok, _ = P.spec_k_topk_logprob_static(big[:, :262144].contiguous(), 4)   # the limit itself is accepted
    torch.cuda.synchronize()
    assert list(ok_tok[0].cpu().numpy()) == [0, 1, 2, 3]               # all-equal logits: lower token ids first
