"""areal_sample_logprob_static (the entry point that allocates nothing: its scratch buffer is
a static device array) against areal_sample_logprob on the same logits: token ids bit for
bit, log-probs to 1e-6 (the same kernels run), on two calls in a row, the second with a
smaller input, so that whatever the first call left in the shared array must not leak into
the second.  Sizes beyond the array are refused with a message and leave the outputs alone."""
import numpy as np
import pytest

from paper_2505_24298_amd import synth

pytestmark = pytest.mark.gpu


def _same(got, want):
    """Token ids equal; log-probs equal to 1e-6 where finite, and -inf in the same places."""
    assert got[0].tolist() == want[0].tolist()
    for g, w in ((got[1], want[1]), (got[2], want[2])):
        fin = np.isfinite(w)
        assert (np.isfinite(g) == fin).all() and (g[~fin] == w[~fin]).all()
        assert np.abs(g[fin] - w[fin]).max(initial=0.0) <= 1e-6


def test_static_scratch_sampler_matches_the_context_entry_point():
    import torch
    from paper_2505_24298_amd import binding
    V = 151936
    eng = binding.Areal(synth.shape("tiny", vocab=V), max_seqs=64, max_seq_len=32, max_batch_tokens=64,
                        kv_blocks=4)
    rng = np.random.default_rng(11)
    first = (rng.standard_normal((100, V)) * 0.8).astype(np.float32)     # 10 work-groups per row
    first[3] *= 8.0
    second = (rng.standard_normal((9, V - 3000)) * 0.8).astype(np.float32)   # fewer rows, fewer segments, 64 per row
    second = np.ascontiguousarray(np.pad(second, ((0, 0), (0, 3000)), constant_values=-30.0))
    for logits, seed in ((first, (7 << 32) | 5), (second, 123)):
        n = logits.shape[0]
        ids = np.arange(n, dtype=np.int32) * 5 + 2
        pos = (np.arange(n, dtype=np.int32) * 104729) % 30000
        dl = torch.from_numpy(logits).cuda()
        d_ids, d_pos = torch.from_numpy(ids).cuda(), torch.from_numpy(pos).cuda()
        for top_p in (1.0, 0.9):
            want = [t.cpu().numpy() for t in eng.sample_logprob(dl, ids, pos, 1.0, top_p, seed)]
            got = [t.cpu().numpy() for t in binding.sample_logprob_static(dl, d_ids, d_pos, 1.0, top_p, seed)]
            _same(got, want)
        forced = torch.from_numpy(rng.integers(0, V - 3000, size=n).astype(np.int32)).cuda()
        want = [t.cpu().numpy() for t in eng.sample_logprob(dl, ids, pos, 1.0, 1.0, seed, forced_tokens=forced)]
        got = [t.cpu().numpy() for t in binding.sample_logprob_static(dl, None, None, 1.0, 1.0, seed,
                                                                      forced_tokens=forced)]
        assert got[0].tolist() == forced.cpu().numpy().tolist()
        _same(got, want)
    # beyond the static array: refused, nothing written
    too_many = torch.zeros((129, 1024), device="cuda")
    out = (torch.full((129,), -7, dtype=torch.int32, device="cuda"), torch.zeros(129, device="cuda"),
           torch.zeros(129, device="cuda"))
    idx = torch.zeros(129, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.ArealError) as e:
        binding.sample_logprob_static(too_many, idx, idx, out=out)
    assert e.value.code == binding.E_NOMEM and "128 rows" in str(e.value)
    assert (out[0] == -7).all()
    with pytest.raises(binding.ArealError) as e:
        binding.sample_logprob_static(torch.zeros((1, 262148), device="cuda"), idx[:1], idx[:1])
    assert e.value.code == binding.E_NOMEM
    with pytest.raises(binding.ArealError) as e:
        binding.sample_logprob_static(too_many[:4], idx[:4], idx[:4], temperature=0.0)
    assert e.value.code == binding.E_INVAL
    eng.close()
