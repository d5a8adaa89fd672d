"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.
The oracle cannot pass over 10^8..10^9 tokens at K = 10^3..10^4 in a test, so:
  - integer work is compared whole: initial topics, phi and n_k after the rebuilds, and the
    whole theta CSR against the oracle's;
  - the sampled assignments are compared on listed tokens the oracle resamples one by one
    (10^7 random picks on C3 and C4, 10^6 on C5: enough to resolve the 10^-6 bound on
    mismatches, plus tokens of the heaviest word, of the longest and of the shortest
    documents), at two states: the first iteration from random topics (densest theta rows)
    and iteration 25 from the GPU's own state after 24 iterations, the regime bench.py times
    (sparser rows, another mix of the sampler's pass shapes);
  - the log-likelihood is the closed form evaluated on the oracle's counts (its recount of
    phi and n_k, its theta CSR), and on C3 also oracle.loglik itself;
  - the invariants sum n_wk = sum n_dk = T, n_k = sum_w n_wk, sum_k n_dk = N_d hold at full size.
Every oracle input is made by the oracle itself (its own Philox initial state) or, for the
later state, is the assignment vector both sides start the compared iteration from."""
import time

import numpy as np
import pytest

import corpus_synth
import oracle

pytestmark = pytest.mark.gpu
SEED = corpus_synth.SAMPLER_SEED
WARM_ITERS = 24          # bench.py: 5 warm-up + 20 timed iterations; the 25th is compared


@pytest.fixture
def say(capfd):
    """Progress lines that reach the terminal while the test runs (a long quiet test looks hung)."""
    t0 = time.time()

    def emit(*a):
        with capfd.disabled():
            print("[%6.1fs] " % (time.time() - t0) + " ".join(str(x) for x in a), flush=True)
    return emit


def need_gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    import paper_1803_04631_amd as mlda
    return mlda


def listed_tokens(c, V, n_listed, rng):
    """Random picks plus the corners: the heaviest word, the longest and the shortest document,
    the first and the last token."""
    T = c.T
    lens = np.diff(c.doc_ptr)
    heavy = int(np.argmax(np.bincount(c.word_ids[:20_000_000], minlength=V)))
    picks = [rng.integers(T, size=n_listed),
             np.flatnonzero(c.word_ids[:2_000_000] == heavy)[:500],
             np.arange(c.doc_ptr[np.argmax(lens)], c.doc_ptr[np.argmax(lens)] + min(lens.max(), 300)),
             np.arange(c.doc_ptr[np.argmin(lens)], c.doc_ptr[np.argmin(lens) + 1]),
             np.array([0, T - 1])]
    return np.unique(np.concatenate(picks)).astype(np.int64)


def closed_form_loglik(cfg, lens, n_wk, n_k, counts):
    """Joint collapsed log-likelihood from counts (phi, n_k, the entries of theta)."""
    from scipy.special import gammaln
    V, K, D = cfg.V, cfg.K, len(lens)

    def entries_term(cells, a):            # sum over positive integer cells of lgG(c + a) - lgG(a)
        nz = cells[cells > 0]
        table = gammaln(np.arange(int(nz.max()) + 1, dtype=np.float64) + a) - gammaln(a)
        return float(np.bincount(nz, minlength=len(table)).astype(np.float64) @ table)

    return (K * gammaln(V * cfg.beta) - gammaln(n_k + V * cfg.beta).sum()
            + entries_term(n_wk, cfg.beta)
            + D * gammaln(K * cfg.alpha) - gammaln(lens + K * cfg.alpha).sum()
            + entries_term(counts, cfg.alpha))


def check_state_after_step(say, name, cfg, c, model, z_before, n_wk, n_k, it, n_listed, theta_docs=None,
                           oracle_loglik=False):
    """`model` has just made iteration `it` from the assignments z_before, whose recount by the
    oracle is (n_wk, n_k).  Compares listed new assignments, then all counts and the
    log-likelihood of the new state."""
    T, V, K = c.T, cfg.V, cfg.K
    D = len(c.doc_ptr) - 1
    lens = np.diff(c.doc_ptr)
    rng = np.random.default_rng(1803 + it)
    z_new = model.assignments()
    assert int(z_new.max()) < K
    tokens = listed_tokens(c, V, n_listed, rng)
    want = oracle.resample_listed(tokens, c.doc_ptr, c.word_ids, z_before, V, K, cfg.alpha, cfg.beta,
                                  SEED, it, n_wk, n_k)
    say(name, "iteration", it, ": oracle resampled", len(tokens), "listed tokens")
    bad = int((z_new[tokens] != want).sum())
    assert bad <= 1e-6 * len(tokens), f"{bad} of {len(tokens)} listed assignments differ"
    del want, tokens

    # counts of the new state: whole recount for phi, whole CSR for theta
    n_wk1, n_k1 = oracle.count_word_topic(c.word_ids, z_new, V, K)
    assert np.array_equal(model.topic_totals(), n_k1)
    g_wk = model.word_topic()
    assert np.array_equal(g_wk, n_wk1)
    assert np.array_equal(g_wk.sum(axis=0, dtype=np.int64), n_k1)          # n_k = sum_w n_wk
    assert int(n_k1.sum(dtype=np.int64)) == T
    del g_wk
    say(name, "phi of the new state matches the recount")
    row_ptr, topics, counts = model.doc_topic_csr()
    assert row_ptr[-1] == model.doc_topic_nnz() == len(counts)
    assert int(counts.sum(dtype=np.int64)) == T                             # sum n_dk = T
    row_sum = np.add.reduceat(counts.astype(np.int64), np.minimum(row_ptr[:-1], len(counts) - 1))
    assert np.array_equal(row_sum[lens > 0], lens[lens > 0])               # Eq. 5
    assert counts.min() > 0 and int(topics.max()) < K
    del row_sum
    if theta_docs is None:
        o_ptr, o_topics, o_counts = oracle.doc_topic_csr(c.doc_ptr, z_new, K)
        assert np.array_equal(row_ptr, o_ptr)
        assert np.array_equal(topics, o_topics)
        assert np.array_equal(counts, o_counts)
        say(name, "whole theta CSR equals the oracle's:", len(o_counts), "entries")
        ll_counts = o_counts
        del o_ptr, o_topics
    else:
        # runs of documents (first, last, around the longest) as corpora of their own
        for lo, hi in theta_docs:
            sub_ptr = c.doc_ptr[lo:hi + 1] - c.doc_ptr[lo]
            o_ptr, o_topics, o_counts = oracle.doc_topic_csr(sub_ptr, z_new[c.doc_ptr[lo]:c.doc_ptr[hi]], K)
            a, b = row_ptr[lo], row_ptr[hi]
            assert np.array_equal(row_ptr[lo:hi + 1] - a, o_ptr)
            assert np.array_equal(topics[a:b], o_topics) and np.array_equal(counts[a:b], o_counts)
        say(name, "theta rows equal the oracle's on", sum(h - l for l, h in theta_docs), "documents")
        ll_counts = counts
    ll = closed_form_loglik(cfg, lens, n_wk1, n_k1, ll_counts)
    got = model.loglik()
    assert abs(got - ll) <= 1e-5 * abs(ll)
    if oracle_loglik:
        ll_o = oracle.loglik(c.doc_ptr, z_new, V, K, cfg.alpha, cfg.beta, n_wk1, n_k1)
        assert abs(got - ll_o) <= 1e-5 * abs(ll_o)
        assert abs(ll - ll_o) <= 1e-9 * abs(ll_o)
    say(name, "log-likelihood agrees:", got / T, "per token")


def check_first_iteration(say, name, cfg, c, n_listed, theta_docs=None, oracle_loglik=False):
    mlda = need_gpu()
    T, V, K = c.T, cfg.V, cfg.K
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
    assert int(n_k.sum(dtype=np.int64)) == T
    model.step(1, loglik=True)
    check_state_after_step(say, name, cfg, c, model, z0, n_wk, n_k, 1, n_listed, theta_docs, oracle_loglik)
    model.close()


def check_later_iteration(say, name, cfg, c, n_listed, oracle_loglik=False):
    """Iteration WARM_ITERS + 1 from the state the GPU itself reached: the assignments are
    downloaded, the oracle recounts them and resamples the listed tokens from there."""
    mlda = need_gpu()
    T, V, K = c.T, cfg.V, cfg.K
    say(name, "generated, T =", T)
    model = mlda.Mlda(c.doc_ptr, c.word_ids, V, K, cfg.alpha, cfg.beta, SEED)
    model.init_random()
    model.step(WARM_ITERS, loglik=True)
    assert model.iteration == WARM_ITERS
    z_before = model.assignments()
    say(name, "state after", WARM_ITERS, "GPU iterations downloaded")
    n_wk, n_k = oracle.count_word_topic(c.word_ids, z_before, V, K)
    assert np.array_equal(model.topic_totals(), n_k)
    assert np.array_equal(model.word_topic(), n_wk)
    say(name, "phi of that state matches the oracle's recount; theta nnz per document",
        model.doc_topic_nnz() / max(1, len(c.doc_ptr) - 1))
    model.step(1, loglik=True)
    check_state_after_step(say, name, cfg, c, model, z_before, n_wk, n_k, WARM_ITERS + 1, n_listed,
                           None, oracle_loglik)
    model.close()


FULL = [("C4", 10_000_000), ("C3", 10_000_000), ("C5", 1_000_000)]


@pytest.mark.parametrize("name,n_listed", FULL)
def test_first_iteration_at_full_size(say, name, n_listed):
    cfg = corpus_synth.CONFIGS[name]
    check_first_iteration(say, name, cfg, corpus_synth.generate(cfg), n_listed, oracle_loglik=(name == "C3"))


@pytest.mark.parametrize("name,n_listed", FULL)
def test_iteration_25_from_the_gpu_state_at_full_size(say, name, n_listed):
    cfg = corpus_synth.CONFIGS[name]
    check_later_iteration(say, name, cfg, corpus_synth.generate(cfg), n_listed, oracle_loglik=(name == "C3"))


def test_first_iteration_near_the_token_limit(say):
    """The library takes fewer than 2^31 tokens: C4's shape with 2.85 times its documents,
    2.1e9 tokens (98 % of the limit), so that token positions, byte offsets beyond 2^32 and
    the slot offsets of 23 million theta rows are exercised near the top of their ranges."""
    cfg = corpus_synth.CONFIGS["C4"]
    c = corpus_synth.generate(cfg, scale=2.85)
    assert 2.05e9 < c.T < 2**31
    D = len(c.doc_ptr) - 1
    longest = int(np.argmax(np.diff(c.doc_ptr)))
    runs = [(0, 200_000), (D - 200_000, D), (max(0, longest - 1000), min(D, longest + 1000)),
            (D // 2, D // 2 + 200_000)]
    check_first_iteration(say, "C4x2.85", cfg, c, 1_000_000, theta_docs=runs)


def test_streamed_chunks_at_full_size(say):
    """C3 cut into three chunks that take turns on the GPU gives, bit for bit, the state the
    resident corpus reaches after two iterations (token indices beyond a chunk's own range,
    chunk boundaries inside the 32-bit position arithmetic, 10^8 tokens through pinned memory)."""
    import torch
    mlda = need_gpu()
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
