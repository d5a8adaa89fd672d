"""Pins for the oracle's count rebuilds, its full pass and its log-likelihood."""
import math

import numpy as np
import pytest

import corpus_synth
import oracle


@pytest.fixture(scope="module")
def small():
    c = corpus_synth.tiny(D=60, V=41, K=7, mean_len=12, seed=3)
    z = oracle.init_topics(c.T, 7, 123)
    return c, z


def doc_of_token(doc_ptr):
    return np.repeat(np.arange(len(doc_ptr) - 1), np.diff(doc_ptr))


def test_word_topic_counts_are_a_recount(small):
    c, z = small
    V, K = c.config.V, c.config.K
    n_wk, n_k = oracle.count_word_topic(c.word_ids, z, V, K)
    brute = np.bincount(c.word_ids.astype(np.int64) * K + z, minlength=V * K).reshape(V, K)
    assert np.array_equal(n_wk, brute)                     # word-major: [v][k], V != K here
    assert np.array_equal(n_k, np.bincount(z, minlength=K))
    assert np.array_equal(n_k, n_wk.sum(axis=0))           # n_k = sum_w n_wk
    assert n_wk.sum() == c.T
    assert np.array_equal(n_wk.sum(axis=1), np.bincount(c.word_ids, minlength=V))


def test_doc_topic_csr_is_canonical(small):
    c, z = small
    K, D = c.config.K, c.config.D
    row_ptr, topics, counts = oracle.doc_topic_csr(c.doc_ptr, z, K)
    dense = np.bincount(doc_of_token(c.doc_ptr) * K + z, minlength=D * K).reshape(D, K)
    assert row_ptr[0] == 0 and row_ptr[-1] == len(topics) == len(counts) == (dense > 0).sum()
    for d in range(D):
        t = topics[row_ptr[d]:row_ptr[d + 1]]; n = counts[row_ptr[d]:row_ptr[d + 1]]
        assert np.all(np.diff(t.astype(int)) > 0) and np.all(n > 0)
        assert np.array_equal(t, np.nonzero(dense[d])[0]) and np.array_equal(n, dense[d][t])
        assert n.sum() == c.doc_ptr[d + 1] - c.doc_ptr[d]      # Eq. 5: DocLen_d = sum_k theta_dk
    assert counts.sum() == c.T


def test_full_pass_is_the_single_token_draw_on_frozen_counts(small):
    """The pass = for every token, the one-token resample fed with rows recounted here
    with numpy, the uniform keyed by (seed, iteration, document-major token index)."""
    c, z = small
    V, K = c.config.V, c.config.K
    alpha, beta, seed, it = 50.0 / K, 0.01, 4631, 3
    z_new = oracle.iteration(c.doc_ptr, c.word_ids, z, V, K, alpha, beta, seed, it, threads=3)
    doc = doc_of_token(c.doc_ptr)
    n_dk = np.bincount(doc * K + z, minlength=c.config.D * K).reshape(-1, K)
    n_wk = np.bincount(c.word_ids.astype(np.int64) * K + z, minlength=V * K).reshape(V, K)
    n_k = np.bincount(z, minlength=K)
    for t in range(c.T):
        want, _, _ = oracle.resample_token(K, V, alpha, beta, n_dk[doc[t]], n_wk[c.word_ids[t]],
                                           n_k, int(z[t]), oracle.uniform(seed, it, t))
        assert z_new[t] == want
    # thread count and the listed-token entry change nothing
    assert np.array_equal(z_new, oracle.iteration(c.doc_ptr, c.word_ids, z, V, K, alpha, beta,
                                                  seed, it, threads=1))
    pick = np.array([0, 5, c.T // 2, c.T - 1])
    n_wk32, n_k32 = oracle.count_word_topic(c.word_ids, z, V, K)
    assert np.array_equal(z_new[pick], oracle.resample_listed(pick, c.doc_ptr, c.word_ids, z, V, K,
                                                              alpha, beta, seed, it, n_wk32, n_k32))
    # another iteration index or seed gives another pass
    assert not np.array_equal(z_new, oracle.iteration(c.doc_ptr, c.word_ids, z, V, K, alpha, beta,
                                                      seed, it + 1))


def chain_rule_loglik(doc_ptr, word_ids, z, V, K, alpha, beta):
    """log p(w, z) as the product of one-step-ahead urn probabilities, token by token."""
    n_kw = np.zeros((K, V)); n_k = np.zeros(K)
    ll = 0.0
    for d in range(len(doc_ptr) - 1):
        n_dk = np.zeros(K)
        for i, t in enumerate(range(doc_ptr[d], doc_ptr[d + 1])):
            k, w = int(z[t]), int(word_ids[t])
            ll += math.log((n_dk[k] + alpha) / (i + K * alpha))
            ll += math.log((n_kw[k, w] + beta) / (n_k[k] + V * beta))
            n_dk[k] += 1; n_kw[k, w] += 1; n_k[k] += 1
    return ll


@pytest.mark.parametrize("D,V,K,alpha,beta", [(3, 5, 3, 0.5, 0.1), (20, 13, 6, 50 / 6, 0.01),
                                              (9, 4, 1, 2.0, 0.3)])
def test_loglik_equals_chain_rule_product(D, V, K, alpha, beta):
    c = corpus_synth.tiny(D=D, V=V, K=K, mean_len=8, seed=D)
    z = oracle.init_topics(c.T, K, 77)
    n_wk, n_k = oracle.count_word_topic(c.word_ids, z, V, K)
    ll = oracle.loglik(c.doc_ptr, z, V, K, alpha, beta, n_wk, n_k)
    want = chain_rule_loglik(c.doc_ptr, c.word_ids, z, V, K, alpha, beta)
    assert abs(ll - want) <= 1e-10 * abs(want)
    if K == 1:      # one topic: the document side is log 1 = 0, only the word urn remains
        n_w = np.bincount(c.word_ids, minlength=V)
        word_only = sum(math.lgamma(n + beta) - math.lgamma(beta) for n in n_w) \
            + math.lgamma(V * beta) - math.lgamma(c.T + V * beta)
        assert abs(ll - word_only) <= 1e-10 * abs(ll)


def test_chain_improves_likelihood_and_sparsifies_theta():
    """Section 7.1: the doc-topic matrix gets sparser over the first iterations; the
    likelihood of the state rises from its random start."""
    c = corpus_synth.tiny(D=300, V=400, K=16, mean_len=60, seed=5, alpha_gen=0.05)
    V, K, alpha, beta = 400, 16, 50 / 16, 0.01
    z = oracle.init_topics(c.T, K, 4631)
    lls, nnzs = [], []
    for it in range(1, 26):
        n_wk, n_k = oracle.count_word_topic(c.word_ids, z, V, K)
        lls.append(oracle.loglik(c.doc_ptr, z, V, K, alpha, beta, n_wk, n_k))
        nnzs.append(oracle.doc_topic_csr(c.doc_ptr, z, K)[0][-1])
        z = oracle.iteration(c.doc_ptr, c.word_ids, z, V, K, alpha, beta, 4631, it, n_wk, n_k)
    assert lls[-1] > lls[0] + 0.05 * abs(lls[0])
    assert nnzs[-1] < 0.9 * nnzs[0]
    # far below the likelihood of the topics the corpus was generated with? No: it must
    # approach it from below or exceed it slightly, never be an order of magnitude off
    n_wk, n_k = oracle.count_word_topic(c.word_ids, c.z_true, V, K)
    ll_true = oracle.loglik(c.doc_ptr, c.z_true, V, K, alpha, beta, n_wk, n_k)
    assert lls[0] < ll_true and lls[-1] > lls[0] + 0.3 * (ll_true - lls[0])
