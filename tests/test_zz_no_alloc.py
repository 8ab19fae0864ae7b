"""GPU test of rollout_sample_static, the sampler entry point that allocates nothing (its
kernels' scratch is a fixed device array inside the library): called through the C ABI on
device arrays, twice in a row - the second call with fewer rows and a smaller vocabulary, so
that it runs over what the first left in the array - and compared with rollout_sample, the
entry point it is a variant of: token ids and integer weight sums bit-exact, log-probs equal."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


def both(logits_np, temperature, top_p, words, forced=None):
    import torch
    import paper_2506_06122_amd as R
    rows, vocab = logits_np.shape
    logits = torch.from_numpy(logits_np).cuda()
    want = R.rollout_sample(logits, temperature, top_p, words, forced=forced)
    uni = torch.from_numpy(words.view(np.int32).copy()).cuda()
    frc = torch.from_numpy(forced).cuda() if forced is not None else None
    toks = torch.full((rows,), -7, dtype=torch.int32, device="cuda")
    lps = torch.full((rows,), float("nan"), dtype=torch.float32, device="cuda")
    sums = torch.full((rows,), -1, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    R.rollout_sample_static(logits, temperature, top_p, uni, toks, lps, forced=frc, weight_sums=sums)
    torch.cuda.synchronize()
    got = (toks.cpu().numpy(), lps.cpu().numpy(), sums.cpu().numpy().view(np.uint64))
    return want, got


def test_static_sampler_matches_the_allocating_one_on_two_calls_in_a_row():
    import paper_2506_06122_amd as R
    # call 1: 12 rows over the large vocabulary (both sweeps split over several workgroups: the
    # partial maxima and segment sums live in the static array); call 2: 5 rows, 40000 ids
    for rows, vocab, top_p, seed in ((12, 151936, 0.9, 1), (5, 40000, 0.3, 2)):
        logits = workloads.random_logits(rows, vocab, seed=seed, scale=2.0)
        logits[0, :] = 0.0
        logits[1, vocab // 3] = 60.0
        words = workloads.uniform_words(rows, seed=seed + 10)
        words[:2] = (0, 2 ** 32 - 1)
        want, got = both(logits, 0.7, top_p, words)
        assert np.array_equal(got[0], want[0]), f"tokens differ at vocab {vocab}"
        assert np.array_equal(got[2], want[2]), "integer weight sums differ"
        assert np.array_equal(got[1], want[1]), "log-probs differ"
    # forced tokens (teacher forcing), a small vocabulary (one workgroup per row, no partial results)
    logits = workloads.random_logits(7, 1000, seed=3, scale=2.0)
    words = workloads.uniform_words(7, seed=4)
    forced = (np.arange(7, dtype=np.int32) * 37) % 1000
    want, got = both(logits, 1.3, 1.0, words, forced=forced)
    assert np.array_equal(got[0], forced) and np.array_equal(want[0], forced)
    assert np.array_equal(got[1], want[1]) and np.array_equal(got[2], want[2])
    # sizes beyond the array are refused with a clear error, nothing runs
    import torch
    big = torch.zeros((R.binding.SAMPLE_STATIC_MAX_ROWS + 1, 64), dtype=torch.float32, device="cuda")
    z = torch.zeros(R.binding.SAMPLE_STATIC_MAX_ROWS + 1, dtype=torch.int32, device="cuda")
    with pytest.raises(R.RolloutError) as e:
        R.rollout_sample_static(big, 1.0, 1.0, z, z.clone(), z.float())
    assert e.value.code == -1 and "ROLLOUT_SAMPLE_STATIC_MAX_ROWS" in str(e.value)
