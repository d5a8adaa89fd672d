"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.
The oracle cannot pass over 10^8..10^9 tokens at K = 10^3..10^4 in a test, so:
  - integer work is compared whole: initial topics, phi and n_k after the rebuilds;
  - the sampled assignments of the first iteration are compared on listed tokens the
    oracle resamples one by one (random picks plus tokens of the heaviest word, of the
    longest and of the shortest documents);
  - theta rows are compared on sampled documents, and the invariants
    sum n_wk = sum n_dk = T, n_k = sum_w n_wk, sum_k n_dk = N_d are checked at full size.
Every oracle input is made by the oracle itself (its own Philox initial state)."""
import os
import time

import numpy as np
import pytest

import corpus_synth
import oracle

pytestmark = pytest.mark.gpu
SEED = corpus_synth.SAMPLER_SEED
_T0 = time.time()


def say(*a):
    line = "[%6.1fs] " % (time.time() - _T0) + " ".join(str(x) for x in a)
    print(line, flush=True)
    try:                                    # keeps a long quiet test visibly alive
        os.makedirs("gpurun_out", exist_ok=True)
        with open("gpurun_out/test_progress.log", "a") as f:
            f.write(line + "\n")
    except OSError:
        pass


@pytest.mark.parametrize("name,n_listed", [("C4", 20000), ("C3", 8000), ("C5", 2500)])
def test_first_iteration_at_full_size(name, n_listed):
    cfg = corpus_synth.CONFIGS[name]
    check_first_iteration(name, cfg, corpus_synth.generate(cfg), n_listed)


def test_first_iteration_near_the_token_limit():
    """The library takes fewer than 2^31 tokens: C4's shape with 2.85 times its documents,
    2.1e9 tokens (98 % of the limit), so that token positions, byte offsets beyond 2^32 and
    the slot offsets of 23 million theta rows are exercised near the top of their ranges."""
    cfg = corpus_synth.CONFIGS["C4"]
    c = corpus_synth.generate(cfg, scale=2.85)
    assert 2.05e9 < c.T < 2**31
    check_first_iteration("C4x2.85", cfg, c, 20000)


def check_first_iteration(name, cfg, c, n_listed):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    import paper_1803_04631_amd as mlda
    T, V, K = c.T, cfg.V, cfg.K
    D = len(c.doc_ptr) - 1
    say(name, "generated, T =", T)
    model = mlda.Mlda(c.doc_ptr, c.word_ids, V, K, cfg.alpha, cfg.beta, SEED)
    model.init_random()
    z0_gpu = model.assignments()
    say(name, "resident, initial topics downloaded")

    z0 = oracle.init_topics(T, K, SEED)
    assert np.array_equal(z0_gpu, z0)
    del z0_gpu
    n_wk, n_k = oracle.count_word_topic(c.word_ids, z0, V, K)
    say(name, "oracle recount done")
    assert np.array_equal(model.topic_totals(), n_k)
    assert np.array_equal(model.word_topic(), n_wk)
    assert int(n_k.sum()) == T

    model.step(1, loglik=True)
    z1 = model.assignments()
    say(name, "one GPU iteration done")
    assert int(z1.max()) < K

    rng = np.random.default_rng(1803)
    lens = np.diff(c.doc_ptr)
    heavy = int(np.argmax(np.bincount(c.word_ids, minlength=V)))
    picks = [rng.integers(T, size=n_listed),
             np.flatnonzero(c.word_ids[:2_000_000] == heavy)[:500],
             np.arange(c.doc_ptr[np.argmax(lens)], c.doc_ptr[np.argmax(lens)] + min(lens.max(), 300)),
             np.arange(c.doc_ptr[np.argmin(lens)], c.doc_ptr[np.argmin(lens) + 1]),
             np.array([0, T - 1])]
    tokens = np.unique(np.concatenate(picks)).astype(np.int64)
    want = oracle.resample_listed(tokens, c.doc_ptr, c.word_ids, z0, V, K, cfg.alpha, cfg.beta,
                                  SEED, 1, n_wk, n_k)
    say(name, "oracle resampled", len(tokens), "listed tokens")
    bad = int((z1[tokens] != want).sum())
    assert bad <= 1e-6 * len(tokens), f"{bad} of {len(tokens)} listed assignments differ"
    del z0, n_wk

    # counts of the new state: whole recount for phi, sampled documents for theta
    n_wk1, n_k1 = oracle.count_word_topic(c.word_ids, z1, V, K)
    assert np.array_equal(model.topic_totals(), n_k1)
    g_wk = model.word_topic()
    assert np.array_equal(g_wk, n_wk1)
    assert np.array_equal(g_wk.sum(axis=0, dtype=np.int64), n_k1)          # n_k = sum_w n_wk
    say(name, "phi of the new state matches the recount")
    del g_wk
    row_ptr, topics, counts = model.doc_topic_csr()
    assert row_ptr[-1] == model.doc_topic_nnz() == len(counts)
    assert int(counts.sum(dtype=np.int64)) == T                             # sum n_dk = T
    row_sum = np.add.reduceat(counts.astype(np.int64), np.minimum(row_ptr[:-1], len(counts) - 1))
    assert np.array_equal(row_sum[lens > 0], lens[lens > 0])               # Eq. 5
    assert counts.min() > 0 and int(topics.max()) < K
    for d in np.concatenate([rng.integers(D, size=300), [0, D - 1, np.argmax(lens)]]):
        row = np.bincount(z1[c.doc_ptr[d]:c.doc_ptr[d + 1]], minlength=K)
        t = topics[row_ptr[d]:row_ptr[d + 1]]
        assert np.array_equal(t, np.flatnonzero(row)) and np.array_equal(counts[row_ptr[d]:row_ptr[d + 1]], row[t])
    say(name, "theta rows match on sampled documents; invariants hold")

    # log-likelihood of the new state: word side in closed form from the recount,
    # document side from the library's own CSR (already checked above)
    from scipy.special import gammaln
    nz = n_wk1[n_wk1 > 0].astype(np.float64)
    ll = (K * gammaln(V * cfg.beta) - gammaln(n_k1 + V * cfg.beta).sum()
          + (gammaln(nz + cfg.beta) - gammaln(cfg.beta)).sum()
          + D * gammaln(K * cfg.alpha) - gammaln(lens + K * cfg.alpha).sum()
          + (gammaln(counts + cfg.alpha) - gammaln(cfg.alpha)).sum())
    assert abs(model.loglik() - ll) <= 1e-5 * abs(ll)
    say(name, "log-likelihood agrees")
    model.close()


def test_streamed_chunks_at_full_size():
    """C3 cut into three chunks that take turns on the GPU gives, bit for bit, the state the
    resident corpus reaches after two iterations (token indices beyond a chunk's own range,
    chunk boundaries inside the 32-bit position arithmetic, 10^8 tokens through pinned memory)."""
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    import paper_1803_04631_amd as mlda
    cfg = corpus_synth.CONFIGS["C3"]
    c = corpus_synth.generate(cfg)
    args = (c.doc_ptr, c.word_ids, cfg.V, cfg.K, cfg.alpha, cfg.beta, SEED)
    resident = mlda.Mlda(*args)
    resident.init_random()
    resident.step(2, loglik=True)
    z, n_k, ll, nnz = resident.assignments(), resident.topic_totals(), resident.loglik(), resident.doc_topic_nnz()
    resident.close()
    del resident
    torch.cuda.empty_cache()
    say("C3 resident run done")
    streamed = mlda.Mlda(*args, chunks=3)
    streamed.init_random()
    streamed.step(2, loglik=True)
    assert streamed.iteration == 2
    assert np.array_equal(streamed.assignments(), z)
    assert np.array_equal(streamed.topic_totals(), n_k)
    assert abs(streamed.loglik() - ll) <= 1e-9 * abs(ll)
    assert streamed.doc_topic_nnz() == nnz
    say("C3 streamed run agrees")
    streamed.close()
