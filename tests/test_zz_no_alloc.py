"""The allocation-free entry point (ad_verify_static) against ad_verify, through the C ABI: two calls in a row on
the library's static scratch, the second with fewer rows, then with a second model on the same GPU in between.
Integer results: bit-exact."""
import numpy as np
import pytest

from paper_2506_03700_amd import synth

pytestmark = pytest.mark.gpu


def test_verify_static_equals_verify():
    import torch
    from paper_2506_03700_amd import binding as ad
    assert torch.cuda.is_available(), "this test needs the GPU"
    shape = synth.MINI8B
    g = ad.Model(shape, synth.make_weights(shape, seed=0), max_pos=16)
    small = synth.TINY.with_(name="tiny-untied", tied_head=False, vocab=301)
    g2 = ad.Model(small, synth.make_weights(small, seed=1), max_pos=16)
    rng = np.random.default_rng(0)
    for m in (6, 3, 8, 1):
        h = torch.from_numpy(synth.make_hidden(shape, seed=30 + m, m=m)).to("cuda:0")
        # drafts: the rows' own final-head tokens, one of them made wrong, so that both outcomes occur
        _, _, arg = g.ad_verify(h, [0] * (m - 1))
        for bad in (None, m // 2):
            draft = [int(x) for x in arg[:m - 1]]
            if bad is not None and m > 1:
                draft[min(bad, m - 2)] = (draft[min(bad, m - 2)] + 1) % shape.vocab
            print(f"case m={m} bad={bad}", flush=True)
            want = g.ad_verify(h, draft)
            got = g.ad_verify(h, draft, static=True)
            # the other model's call leaves its own partials in the shared array
            h2 = torch.from_numpy(synth.make_hidden(small, seed=m, m=2)).to("cuda:0")
            want2 = g2.ad_verify(h2, [int(rng.integers(0, small.vocab))])
            got2 = g2.ad_verify(h2, [want2[2][0]], static=True)
            assert got2[2].tolist() == want2[2].tolist()
            again = g.ad_verify(h, draft, static=True)
            for r in (got, again):
                assert (r[0], r[1]) == (want[0], want[1]) and r[2].tolist() == want[2].tolist()
    g.close()
    g2.close()
