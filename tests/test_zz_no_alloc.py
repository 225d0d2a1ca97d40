"""The entry point that allocates nothing (mtp_subset_build_static: scratch in an array built into the library) against
the entry point it is a variant of (mtp_subset_build with a caller's workspace): counts, list and skipped-id count
bit-exact (integer work), on two calls in a row, the second with a smaller input; a vocabulary beyond the built-in
scratch is refused.  Outputs are allocated before the calls; the calls themselves go straight through the C ABI."""
import numpy as np
import pytest

from paper_2509_18362_amd import synth

pytestmark = pytest.mark.gpu


def test_static_scratch_list_builder_matches_workspace_entry_point():
    import torch
    assert torch.cuda.is_available()
    from paper_2509_18362_amd import binding
    dev = "cuda:0"
    vmax = binding.mtp_subset_static_max_vocab()
    assert vmax >= synth.SEVEN_B.vocab_size
    cases = [(synth.SEVEN_B.vocab_size, (1 << 22) + 3, 32768, 11), (4096, (1 << 16) + 1, 819, 12)]
    for V, N, n, seed in cases:  # the second call is smaller in every dimension: stale scratch would show
        toks = torch.from_numpy(synth.make_token_stream(V, N, seed=seed, invalid_every=997)).to(dev)
        want = binding.build_subset(toks, V, n, want_counts=True)
        ids = torch.full((n,), -7, dtype=torch.int32, device=dev)
        counts = torch.full((V,), -7, dtype=torch.int32, device=dev)
        invalid = torch.full((4,), -7, dtype=torch.int32, device=dev)
        torch.cuda.synchronize()
        st = binding.mtp_subset_build_static(toks, toks.numel(), V, n, ids, counts, invalid,
                                             torch.cuda.current_stream().cuda_stream)
        assert st == 0
        torch.cuda.synchronize()
        np.testing.assert_array_equal(counts.cpu().numpy(), want["counts"].cpu().numpy())
        np.testing.assert_array_equal(ids.cpu().numpy(), want["ids"].cpu().numpy())
        assert int(invalid.cpu().numpy()[0]) == int(want["invalid"].cpu().numpy()[0]) > 0
    # beyond the built-in scratch: refused on the host, nothing enqueued
    big = torch.zeros(16, dtype=torch.int32, device=dev)
    assert binding.mtp_subset_build_static(big, 16, vmax + 1, 4, big, None, None, 0) == -7
    assert binding.mtp_subset_build_static(None, 16, 100, 4, big, None, None, 0) == -1
