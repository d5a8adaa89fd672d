"""The synthetic corpora have the shapes the paper's workloads have (Table 3, Section 7.1)."""
import numpy as np

import corpus_synth as cs


def test_named_configs_match_paper_shapes(golden):
    for name, tokens, docs, words, mean_len in golden("table3_dataset_shapes.txt"):
        cfg = cs.CONFIGS[name]
        assert abs(cfg.D - int(docs)) <= 0.001 * int(docs)
        assert abs(cfg.V - int(words)) <= 0.004 * int(words)
        scale = 0.02 if name == "C4" else 0.2
        c = cs.generate(name, scale=scale)
        lens = np.diff(c.doc_ptr)
        assert lens.min() >= 1
        assert abs(lens.mean() * cfg.D - int(tokens)) <= 0.02 * int(tokens)       # T within 2 %
        assert abs(lens.mean() - float(mean_len)) <= 0.03 * float(mean_len)
    assert cs.CONFIGS["C5"].K == 10_000 and cs.CONFIGS["C5"].D == cs.CONFIGS["C3"].D


def test_small_configs():
    c1 = cs.generate("C1")
    assert abs(c1.T - 100_000) < 2_000 and c1.word_ids.dtype == np.int32
    assert c1.doc_ptr.dtype == np.int64 and c1.z_true.dtype == np.uint16
    assert c1.word_ids.min() >= 0 and c1.word_ids.max() < 5_000 and c1.z_true.max() < 32
    assert cs.CONFIGS["C1"].alpha == 50 / 32 and cs.CONFIGS["C1"].beta == 0.01


def test_seeded_and_thread_invariant():
    a = cs.generate("C1", threads=1); b = cs.generate("C1", threads=5)
    assert np.array_equal(a.word_ids, b.word_ids) and np.array_equal(a.z_true, b.z_true)
    c = cs.generate("C1", seed=99)
    assert not np.array_equal(a.word_ids[:1000], c.word_ids[:1000])


def test_word_frequencies_are_heavy_tailed_and_ids_shuffled():
    c = cs.generate("C2")
    freq = np.sort(np.bincount(c.word_ids, minlength=c.config.V))[::-1]
    assert freq[0] > 0.05 * c.T                 # Zipf head
    assert freq[100] < 0.02 * freq[0]
    top = np.argsort(np.bincount(c.word_ids, minlength=c.config.V))[::-1][:50]
    assert not np.array_equal(top, np.arange(50))           # id is not the frequency rank


def test_documents_are_topically_sparse():
    c = cs.generate("C2")
    doc = np.repeat(np.arange(c.config.D), np.diff(c.doc_ptr))
    nnz = len(np.unique(doc.astype(np.int64) * c.config.K + c.z_true)) / c.config.D
    assert nnz < 0.6 * np.diff(c.doc_ptr).mean()


def test_poisson_lengths_of_large_mean():
    """Document lengths follow the requested mean also where exp(-mean) underflows (a
    product-of-uniforms sampler alone would stop near 745 tokens)."""
    for mean in (300.0, 2000.0, 17000.0):
        c = cs.tiny(D=200, V=50, K=8, mean_len=mean, seed=11)
        lens = np.diff(c.doc_ptr)
        # Poisson: mean and variance both equal `mean`; 200 documents
        assert abs(lens.mean() - mean) < 5 * np.sqrt(mean / 200)
        assert 0.6 * mean < lens.var() < 1.5 * mean
