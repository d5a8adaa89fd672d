"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Bars: integer work (initial topics, counts, CSR rows) bit-exact;
sampled assignments may differ from the oracle on at most 1e-6 of the tokens (fp64
rounding order at a CDF boundary); log-likelihood within 1e-5 relative."""
import ctypes

import numpy as np
import pytest

import corpus_synth
import oracle

pytestmark = pytest.mark.gpu

Z_MISMATCH_FRACTION = 1e-6
LL_RTOL = 1e-5
SEED = corpus_synth.SAMPLER_SEED


@pytest.fixture(scope="module")
def mlda():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need a real MI355X")
    import paper_1803_04631_amd as m
    m.load_library()
    return m


def say(*a):
    print(*a, flush=True)


def check_counts(model, c, z, V, K):
    """Counts held by the library == a recount of z by the oracle (bit-exact)."""
    n_wk, n_k = oracle.count_word_topic(c.word_ids, z, V, K)
    assert np.array_equal(model.word_topic(), n_wk)
    assert np.array_equal(model.topic_totals(), n_k)
    row_ptr, topics, counts = oracle.doc_topic_csr(c.doc_ptr, z, K)
    g_ptr, g_top, g_cnt = model.doc_topic_csr()
    assert np.array_equal(g_ptr, row_ptr)
    assert np.array_equal(g_top, topics)
    assert np.array_equal(g_cnt, counts)
    assert model.doc_topic_nnz() == row_ptr[-1]
    assert n_wk.sum() == counts.sum() == len(z) and n_k.sum() == len(z)
    return n_wk, n_k


def check_step(model, c, z, V, K, alpha, beta, seed, it):
    """One iteration from state z on both sides; returns the GPU's new state."""
    n_wk, n_k = oracle.count_word_topic(c.word_ids, z, V, K)
    want = oracle.iteration(c.doc_ptr, c.word_ids, z, V, K, alpha, beta, seed, it, n_wk, n_k)
    model.step(1)
    got = model.assignments()
    assert got.max(initial=0) < K
    bad = int((got != want).sum())
    assert bad <= Z_MISMATCH_FRACTION * len(z), f"{bad} of {len(z)} assignments differ at iteration {it}"
    n_wk2, n_k2 = check_counts(model, c, got, V, K)
    ll = oracle.loglik(c.doc_ptr, got, V, K, alpha, beta, n_wk2, n_k2)
    assert abs(model.loglik() - ll) <= LL_RTOL * abs(ll)
    return got


def test_philox_bitwise(mlda):
    n = 1 << 20
    for seed, it, t0 in [(SEED, 1, 0), (2**63 + 12345, 77, 2**32 - 1000), (0, 0, 2**40)]:
        say("philox", seed, it, t0)
        got = mlda.philox_uniform(seed, it, t0, n).cpu().numpy()
        assert np.array_equal(got, oracle.uniforms(seed, it, t0, n))


@pytest.mark.parametrize("name,iters", [("C1", 10), ("C2", 6)])
def test_named_config_free_running(mlda, name, iters):
    """Configs C1 and C2: initial state, then every iteration, against the oracle."""
    c = corpus_synth.generate(name)
    cfg = c.config
    say(name, "T", c.T)
    model = mlda.Mlda(c.doc_ptr, c.word_ids, cfg.V, cfg.K, cfg.alpha, cfg.beta, SEED)
    model.init_random()
    z = oracle.init_topics(c.T, cfg.K, SEED)
    assert np.array_equal(model.assignments(), z)
    check_counts(model, c, z, cfg.V, cfg.K)
    nnz = [model.doc_topic_nnz()]
    for it in range(1, iters + 1):
        say(name, "iteration", it)
        z = check_step(model, c, z, cfg.V, cfg.K, cfg.alpha, cfg.beta, SEED, it)
        nnz.append(model.doc_topic_nnz())
        assert model.iteration == it
    assert nnz[-1] < nnz[0]          # Section 7.1: theta gets sparser over the first iterations
    model.close()


def test_converged_like_state(mlda):
    """Start from the topics the corpus was generated with (sparse theta rows)."""
    c = corpus_synth.generate("C2")
    cfg = c.config
    model = mlda.Mlda(c.doc_ptr, c.word_ids, cfg.V, cfg.K, cfg.alpha, cfg.beta, SEED)
    model.set_assignments(c.z_true, it=40)
    assert model.iteration == 40
    assert np.array_equal(model.assignments(), c.z_true)
    check_counts(model, c, c.z_true, cfg.V, cfg.K)
    check_step(model, c, c.z_true, cfg.V, cfg.K, cfg.alpha, cfg.beta, SEED, 41)
    model.close()


EDGE_CASES = [
    # name,                 D,   V,    K,   mean_len
    ("single_topic",        50,  30,   1,   10),
    ("two_topics",          50,  30,   2,   10),
    ("k_not_mult_of_16",    80,  60,   37,  30),
    ("k_just_over_wave",    60,  90,   65,  300),     # rows longer than one wave
    ("long_rows",           40,  500,  300, 2500),    # nnz up to ~300: several row chunks
    ("one_word_vocab",      40,  1,    8,   20),
    ("large_k_small_docs",  300, 2000, 10000, 120),   # C5-like K: 45 KB of LDS per tile
    ("short_docs",          3000, 200, 16,  1.2),     # many single-token documents (S = 0)
    # large K, words of every size: several tiles, one tile of more than 1024 tokens, and
    # small ones, which one workgroup takes in runs of 16 (p* of a word derived from the word before)
    ("large_k_mixed_words", 400, 70,   3000, 300),
    ("k_twenty_thousand",   40,  300,  20000, 400),   # every kernel beyond 64 KB of LDS
    ("k_near_lds_limit",    40,  300,  30800, 400),   # 160 KB of LDS: one workgroup per CU
    # K whose p* does not fit a workgroup's LDS: p* of a tile in device memory, a fixed number of
    # workgroups that take tile after tile (1,500 words: more tiles than workgroups); beyond
    # 32,768 topics the histograms of phi and n_k are taken in two ranges of topics
    ("k_beyond_lds",         40,  300,  31000, 400),
    ("k_beyond_lds_many_words", 200, 1500, 33000, 40),
    ("k_largest",            30,  200,  65535, 300),
    # long documents over few topics: counts far beyond one entry's field are spread over
    # several entries of the same topic (2-byte entries hold counts up to 15)
    ("huge_docs_split_rows", 3,   400,  700, 17000),
    ("huge_docs_few_topics", 4,   50,   24,  16500),
    # rows too long for the kept pass shapes: walked twice by a whole wave (4-byte and 2-byte entries)
    ("rows_over_768",        6,   300,  1200, 9000),
    ("rows_over_768_split",  3,   300,  1100, 17500),
    ("rows_near_k_tiny",     3,   300,  1023, 30000),     # the largest K of the 2-byte entries
    ("k_first_packed",       30,  300,  1024, 400),       # the smallest K of the 4-byte entries
]


@pytest.mark.parametrize("case", EDGE_CASES, ids=[c[0] for c in EDGE_CASES])
def test_edge_shapes(mlda, case):
    name, D, V, K, mean_len = case
    c = corpus_synth.tiny(D=D, V=V, K=K, mean_len=mean_len, seed=len(name), name=name)
    alpha, beta = 50.0 / K, 0.01
    say(name, "T", c.T)
    model = mlda.Mlda(c.doc_ptr, c.word_ids, V, K, alpha, beta, SEED)
    model.init_random()
    z = oracle.init_topics(c.T, K, SEED)
    assert np.array_equal(model.assignments(), z)
    for it in (1, 2, 3):
        z = check_step(model, c, z, V, K, alpha, beta, SEED, it)
    model.close()


@pytest.mark.parametrize("case", [("tiny_rows", 60, 90, 65, 300), ("packed_rows", 30, 300, 1024, 400),
                                  ("packed_rows_long_docs", 3, 300, 1100, 17500),
                                  ("large_k", 300, 2000, 10000, 120), ("k_beyond_lds", 40, 300, 31000, 400)],
                         ids=lambda c: c[0])
def test_wide_slot_offsets(mlda, case, monkeypatch):
    """The sampler kernels that address theta rows with 64-bit offsets (what rows beyond 4 GiB
    need; the full-size test of 2.1e9 tokens reaches only one of them), on small inputs."""
    name, D, V, K, mean_len = case
    monkeypatch.setenv("MLDA_WIDE_SLOT_OFFSETS", "1")
    c = corpus_synth.tiny(D=D, V=V, K=K, mean_len=mean_len, seed=len(name), name=name)
    alpha, beta = 50.0 / K, 0.01
    model = mlda.Mlda(c.doc_ptr, c.word_ids, V, K, alpha, beta, SEED)
    model.init_random()
    z = oracle.init_topics(c.T, K, SEED)
    for it in (1, 2):
        z = check_step(model, c, z, V, K, alpha, beta, SEED, it)
    model.close()


def test_long_document_with_more_topics_than_32bit_counters_fit(mlda):
    """A document of 2^16 tokens or more needs 32-bit counters in the theta rebuild; beyond
    32,768 topics they do not fit the LDS at once and the document is counted in two ranges of
    topics, its row growing range by range.  Counts beyond one entry's 16,383 in both ranges."""
    V, K = 50, 40000
    lens = np.array([70000, 300, 5, 0, 66000], dtype=np.int64)
    doc_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    rng = np.random.default_rng(5)
    words = rng.integers(V, size=int(lens.sum())).astype(np.int32)
    z = rng.integers(K, size=len(words)).astype(np.uint16)
    z[0:20000] = 7                              # 20,000 tokens of a topic of the first range
    z[20000:38000] = 32767                      # the last topic of the first range
    z[38000:56000] = 32768                      # the first topic of the second
    z[56000:60000] = K - 1
    z[doc_ptr[4]:doc_ptr[4] + 40000] = 39000    # the last document: mostly one topic of the second range

    class C:  # minimal corpus record
        pass
    c = C(); c.doc_ptr = doc_ptr; c.word_ids = words; c.T = len(words)
    alpha, beta = 50.0 / K, 0.01
    model = mlda.Mlda(doc_ptr, words, V, K, alpha, beta, SEED)
    model.set_assignments(z, it=0)
    assert np.array_equal(model.assignments(), z)
    check_counts(model, c, z, V, K)
    check_step(model, c, z, V, K, alpha, beta, SEED, 1)
    model.close()


@pytest.mark.parametrize("K", [500, 1500])
def test_counts_beyond_one_entry(mlda, K):
    """Documents whose tokens sit in one or two topics: counts of 20,000 to 70,000, which no entry
    of a theta row holds (15 with 2-byte entries, K = 500; 16,383 with 4-byte entries, K = 1500),
    so that a topic takes several entries in a row, also across the lanes of the row walk; a
    document of 2^16 tokens or more needs 32-bit counters in the rebuild."""
    V = 60
    lens = np.array([70000, 40000, 20000, 300, 17, 1, 16384, 15, 16], dtype=np.int64)
    doc_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    rng = np.random.default_rng(K)
    words = rng.integers(V, size=int(lens.sum())).astype(np.int32)
    z = rng.integers(K, size=len(words)).astype(np.uint16)
    z[doc_ptr[0]:doc_ptr[1]] = 3                                   # one topic
    z[doc_ptr[1]:doc_ptr[1] + 20000] = 0                           # two topics, at both ends of a row
    z[doc_ptr[1] + 20000:doc_ptr[2]] = K - 1
    z[doc_ptr[2]:doc_ptr[3]] = rng.integers(5, size=20000) * 7     # five topics
    z[doc_ptr[6]:doc_ptr[7]] = 11                                  # exactly 2^14 tokens of one topic
    z[doc_ptr[7]:doc_ptr[8]] = 2                                   # exactly 15
    z[doc_ptr[8]:doc_ptr[9]] = 2                                   # exactly 16

    class C:  # minimal corpus record
        pass
    c = C(); c.doc_ptr = doc_ptr; c.word_ids = words; c.T = len(words)
    alpha, beta = 50.0 / K, 0.01
    model = mlda.Mlda(doc_ptr, words, V, K, alpha, beta, SEED)
    model.set_assignments(z, it=0)
    assert np.array_equal(model.assignments(), z)
    check_counts(model, c, z, V, K)
    for it in (1, 2):
        z = check_step(model, c, z, V, K, alpha, beta, SEED, it)
    model.close()


def test_mixed_row_lengths(mlda):
    """Documents of 3 to ~1500 tokens over few words: every group width and quad count of the
    row walk occurs, and the 64 tokens a wave takes together mix several of them."""
    V, K = 24, 2000
    parts = [corpus_synth.tiny(D=5, V=V, K=K, mean_len=m, seed=int(m), name="part")
             for m in (3, 12, 28, 45, 75, 110, 170, 300, 600, 1000, 1500)]
    lens = np.concatenate([np.diff(p.doc_ptr) for p in parts])
    order = np.random.default_rng(5).permutation(len(lens))          # lengths in no order
    starts = np.concatenate([[0], np.cumsum(lens)])
    words_by_doc = np.concatenate([p.word_ids for p in parts])
    words = np.concatenate([words_by_doc[starts[d]:starts[d + 1]] for d in order]).astype(np.int32)
    doc_ptr = np.concatenate([[0], np.cumsum(lens[order])]).astype(np.int64)

    class C:  # minimal corpus record
        pass
    c = C(); c.doc_ptr = doc_ptr; c.word_ids = words; c.T = len(words)
    alpha, beta = 50.0 / K, 0.01
    say("mixed_row_lengths T", c.T, "longest", lens.max())
    model = mlda.Mlda(doc_ptr, words, V, K, alpha, beta, SEED)
    model.init_random()
    z = oracle.init_topics(c.T, K, SEED)
    nnz = np.diff(model.doc_topic_csr()[0])
    assert nnz.min() <= 16 and nnz.max() > 768      # from the narrowest shape to the widest
    for it in (1, 2, 3):
        z = check_step(model, c, z, V, K, alpha, beta, SEED, it)
    model.close()


def test_empty_documents_and_unused_words(mlda):
    base = corpus_synth.tiny(D=30, V=40, K=12, mean_len=9, seed=2)
    lens = np.diff(base.doc_ptr)
    # interleave empty documents, keep the same tokens; shift word ids so that word 0
    # and the last words never occur
    new_lens = np.zeros(2 * len(lens) + 3, dtype=np.int64)
    new_lens[1:2 * len(lens):2] = lens
    doc_ptr = np.concatenate([[0], np.cumsum(new_lens)]).astype(np.int64)
    words = (base.word_ids + 1).astype(np.int32)
    V, K, alpha, beta = 50, 12, 0.7, 0.05

    class C:  # minimal corpus record
        pass
    c = C(); c.doc_ptr = doc_ptr; c.word_ids = words; c.T = len(words)
    model = mlda.Mlda(doc_ptr, words, V, K, alpha, beta, 9)
    model.init_random()
    z = oracle.init_topics(c.T, K, 9)
    for it in (1, 2):
        z = check_step(model, c, z, V, K, alpha, beta, 9, it)
    n_wk = model.word_topic()
    assert n_wk[0].sum() == 0 and n_wk[41:].sum() == 0
    model.close()


@pytest.mark.parametrize("chunks", [2, 3, 7])
def test_streamed_chunks_match_oracle(mlda, chunks):
    """The corpus cut into chunks that take turns on the GPU (Algorithm 1, WorkSchedule2) gives
    the oracle's results like the resident corpus does."""
    c = corpus_synth.generate("C1")
    cfg = c.config
    model = mlda.Mlda(c.doc_ptr, c.word_ids, cfg.V, cfg.K, cfg.alpha, cfg.beta, SEED, chunks=chunks)
    model.init_random()
    z = oracle.init_topics(c.T, cfg.K, SEED)
    assert np.array_equal(model.assignments(), z)
    check_counts(model, c, z, cfg.V, cfg.K)
    for it in (1, 2, 3):
        say("streamed", chunks, "iteration", it)
        z = check_step(model, c, z, cfg.V, cfg.K, cfg.alpha, cfg.beta, SEED, it)
    # the log-likelihood evaluated inside the step, and two iterations in one call
    model.step(2, loglik=True)
    for it in (4, 5):
        n_wk, n_k = oracle.count_word_topic(c.word_ids, z, cfg.V, cfg.K)
        z = oracle.iteration(c.doc_ptr, c.word_ids, z, cfg.V, cfg.K, cfg.alpha, cfg.beta, SEED, it, n_wk, n_k)
    assert model.iteration == 5 and np.array_equal(model.assignments(), z)
    n_wk, n_k = check_counts(model, c, z, cfg.V, cfg.K)
    ll = oracle.loglik(c.doc_ptr, z, cfg.V, cfg.K, cfg.alpha, cfg.beta, n_wk, n_k)
    assert abs(model.loglik() - ll) <= LL_RTOL * abs(ll)
    ms, moved = model.timing(), model.sampler_bytes()      # per iteration, summed over the chunks
    assert ms.shape == (2, 4) and np.all(ms > 0) and moved.shape == (2,)
    assert np.all(moved >= 16.0 * c.T)
    model.close()


def test_streamed_with_weights_in_device_memory(mlda):
    """K beyond the LDS column, the corpus in three chunks: p* in device memory, phi counted in
    two ranges of topics and added to chunk by chunk."""
    D, V, K = 30, 100, 33000
    c = corpus_synth.tiny(D=D, V=V, K=K, mean_len=100, seed=8, name="far_streamed")
    alpha, beta = 50.0 / K, 0.01
    model = mlda.Mlda(c.doc_ptr, c.word_ids, V, K, alpha, beta, SEED, chunks=3)
    model.init_random()
    z = oracle.init_topics(c.T, K, SEED)
    for it in (1, 2):
        z = check_step(model, c, z, V, K, alpha, beta, SEED, it)
    model.close()


def test_streamed_edge_cases(mlda):
    """More chunks than documents, empty documents, long documents over few topics, and a saved
    state carried from a resident context into a streamed one."""
    base = corpus_synth.tiny(D=5, V=30, K=9, mean_len=12, seed=3)
    lens = np.diff(base.doc_ptr)
    new_lens = np.zeros(2 * len(lens) + 1, dtype=np.int64)
    new_lens[1::2] = lens                                   # empty documents in between

    class C:  # minimal corpus record
        pass
    c = C(); c.doc_ptr = np.concatenate([[0], np.cumsum(new_lens)]).astype(np.int64)
    c.word_ids = base.word_ids; c.T = base.T
    V, K, alpha, beta = 30, 9, 0.4, 0.02
    model = mlda.Mlda(c.doc_ptr, c.word_ids, V, K, alpha, beta, 11, chunks=16)
    model.init_random()
    z = oracle.init_topics(c.T, K, 11)
    for it in (1, 2):
        z = check_step(model, c, z, V, K, alpha, beta, 11, it)
    model.close()

    big = corpus_synth.tiny(D=4, V=40, K=50, mean_len=16500, seed=8)      # counts spread over many entries
    model = mlda.Mlda(big.doc_ptr, big.word_ids, 40, 50, 1.0, 0.01, SEED, chunks=3)
    model.init_random()
    z = oracle.init_topics(big.T, 50, SEED)
    z = check_step(model, big, z, 40, 50, 1.0, 0.01, SEED, 1)
    model.close()

    c1 = corpus_synth.generate("C1")
    cfg = c1.config
    args = (c1.doc_ptr, c1.word_ids, cfg.V, cfg.K, cfg.alpha, cfg.beta, SEED)
    a = mlda.Mlda(*args); a.init_random(); a.step(4)
    r = mlda.Mlda(*args); r.init_random(); r.step(2)
    s = mlda.Mlda(*args, chunks=4); s.set_assignments(r.assignments(), it=r.iteration); s.step(2)
    assert np.array_equal(s.assignments(), a.assignments())
    assert np.array_equal(s.word_topic(), a.word_topic())
    assert abs(s.loglik() - a.loglik()) <= 1e-9 * abs(a.loglik())
    for m in (a, r, s):
        m.close()

    empty = mlda.Mlda(np.zeros(3, dtype=np.int64), np.zeros(0, dtype=np.int32), 4, 3, 0.5, 0.01, 1, chunks=2)
    empty.init_random(); empty.step(2, loglik=True)
    assert empty.iteration == 2 and empty.doc_topic_nnz() == 0 and abs(empty.loglik()) < 1e-9
    empty.close()


def test_phi_cell_widths(mlda):
    """phi keeps 16-bit cells for words with fewer than 2^16 tokens and int32 rows for the
    others: words with 65535, 65536 and 70001 tokens, every token of a word on one topic (the
    largest value a 16-bit cell can take, and the first that needs the wide row), an odd K so
    that rows start in the middle of a dword; resident and streamed (cells added to by
    several chunks)."""
    V, K, alpha, beta = 5, 7, 0.5, 0.01
    word_counts = np.array([65535, 65536, 70001, 10, 0])
    rng = np.random.default_rng(5)
    word_ids = rng.permutation(np.repeat(np.arange(V, dtype=np.int32), word_counts))
    T = len(word_ids)
    lens = rng.multinomial(T, np.ones(400) / 400).astype(np.int64)

    class C:
        pass
    c = C(); c.word_ids = word_ids; c.T = T
    c.doc_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    z_one = (c.word_ids % K).astype(np.uint16)              # word v entirely on topic v
    for chunks in (1, 3):
        say("phi cell widths, chunks", chunks)
        model = mlda.Mlda(c.doc_ptr, c.word_ids, V, K, alpha, beta, SEED, chunks=chunks)
        model.set_assignments(z_one, it=0)
        n_wk, _ = check_counts(model, c, z_one, V, K)
        assert n_wk[0, 0] == 65535 and n_wk[1, 1] == 65536 and n_wk[2, 2] == 70001
        n_wk, n_k = oracle.count_word_topic(c.word_ids, z_one, V, K)
        ll = oracle.loglik(c.doc_ptr, z_one, V, K, alpha, beta, n_wk, n_k)
        assert abs(model.loglik() - ll) <= LL_RTOL * abs(ll)
        z = z_one
        for it in (1, 2):
            z = check_step(model, c, z, V, K, alpha, beta, SEED, it)
        model.close()


def test_empty_corpus(mlda):
    doc_ptr = np.zeros(4, dtype=np.int64)
    model = mlda.Mlda(doc_ptr, np.zeros(0, dtype=np.int32), 5, 3, 0.5, 0.01, 1)
    model.init_random()
    model.step(2)
    assert model.iteration == 2 and len(model.assignments()) == 0
    assert model.word_topic().sum() == 0 and model.doc_topic_nnz() == 0
    row_ptr, topics, counts = model.doc_topic_csr()
    assert np.array_equal(row_ptr, np.zeros(4)) and len(topics) == 0
    # all counts zero: every lgamma difference vanishes
    assert abs(model.loglik()) < 1e-9
    model.close()


def test_deterministic_and_resumable(mlda):
    """Two runs are bit-identical; 6 iterations == 3 + export + new context + import + 3."""
    c = corpus_synth.generate("C1")
    cfg = c.config
    args = (c.doc_ptr, c.word_ids, cfg.V, cfg.K, cfg.alpha, cfg.beta, SEED)
    a = mlda.Mlda(*args); a.init_random(); a.step(6)
    b = mlda.Mlda(*args); b.init_random(); b.step(6)
    za = a.assignments()
    assert np.array_equal(za, b.assignments())
    assert a.loglik() == b.loglik()
    r = mlda.Mlda(*args); r.init_random(); r.step(3)
    saved, it = r.assignments(), r.iteration
    r.close()
    r2 = mlda.Mlda(*args); r2.set_assignments(saved, it=it); r2.step(3)
    assert np.array_equal(r2.assignments(), za) and r2.iteration == 6
    assert np.array_equal(r2.word_topic(), a.word_topic())
    # another seed is another chain
    d = mlda.Mlda(*args[:-1], SEED + 1); d.init_random(); d.step(1)
    assert not np.array_equal(d.assignments()[:1000], za[:1000])
    for m in (a, b, r2, d):
        m.close()


def test_step_with_loglik_flag_and_timing(mlda):
    c = corpus_synth.generate("C1")
    cfg = c.config
    model = mlda.Mlda(c.doc_ptr, c.word_ids, cfg.V, cfg.K, cfg.alpha, cfg.beta, SEED)
    model.init_random()
    ll0 = model.loglik()
    model.step(4, loglik=True)
    ms = model.timing()
    assert ms.shape == (4, 4) and np.all(ms[:, :3] > 0) and np.all(ms < 1000)
    z = model.assignments()
    n_wk, n_k = oracle.count_word_topic(c.word_ids, z, cfg.V, cfg.K)
    ll = oracle.loglik(c.doc_ptr, z, cfg.V, cfg.K, cfg.alpha, cfg.beta, n_wk, n_k)
    assert abs(model.loglik() - ll) <= LL_RTOL * abs(ll)
    assert model.loglik() > ll0
    # the algorithmic byte count of each launch follows its definition: the state a launch
    # samples from is the one before it
    per_word = np.bincount(c.word_ids, minlength=cfg.V)
    n_tiles = int(np.ceil(per_word / 1024).sum())
    n_wide_tiles = int(np.ceil(per_word[per_word >= 2**16] / 1024).sum())   # int32 rows of phi
    lens = np.diff(c.doc_ptr)

    def row_entries(assignments):
        """Entries of every theta row: K < 1024 gives 2-byte entries that hold counts up to 15,
        so a larger count takes several."""
        row_ptr, _, counts = oracle.doc_topic_csr(c.doc_ptr, assignments, cfg.K)
        per_topic = -(-counts.astype(np.int64) // 15)
        return np.array([per_topic[row_ptr[d]:row_ptr[d + 1]].sum() for d in range(len(lens))])

    assert cfg.K < 1024
    before = row_entries(model.assignments())
    model.step(2)
    mid = row_entries(oracle.iteration(c.doc_ptr, c.word_ids, z, cfg.V, cfg.K, cfg.alpha, cfg.beta, SEED, 5))
    got = model.sampler_bytes()
    assert (before > np.diff(oracle.doc_topic_csr(c.doc_ptr, z, cfg.K)[0])).any()     # some counts are spread
    for entries, b in zip((before, mid), got):
        want = (16.0 * c.T + 2.0 * float((lens * entries).sum())
                + cfg.K * (2.0 * n_tiles + 2.0 * n_wide_tiles))
        assert b == want
    assert len(got) == 2
    model.close()


def test_sampler_bytes_with_runs_of_small_words(mlda):
    """K > 2048: the words of at most 1024 tokens are sampled in runs of 16 and count 6 bytes per
    token instead of a row of phi each, but for the first word of every run."""
    D, V, K = 300, 500, 4000
    c = corpus_synth.tiny(D=D, V=V, K=K, mean_len=200, seed=21, name="runs")
    alpha, beta = 50.0 / K, 0.01
    model = mlda.Mlda(c.doc_ptr, c.word_ids, V, K, alpha, beta, SEED)
    model.init_random()
    z = oracle.init_topics(c.T, K, SEED)
    z = check_step(model, c, z, V, K, alpha, beta, SEED, 1)
    row_ptr, _, _ = oracle.doc_topic_csr(c.doc_ptr, oracle.init_topics(c.T, K, SEED), K)
    lens = np.diff(c.doc_ptr)
    per_word = np.bincount(c.word_ids, minlength=V)
    per_word = per_word[per_word > 0]
    n_tiles = int(np.ceil(per_word / 4096).sum())
    in_runs = per_word[per_word <= 1024]
    assert 16 < len(in_runs) < len(per_word)          # runs, and words outside them
    staged_rows = n_tiles - len(in_runs) + -(-len(in_runs) // 16)
    want = (16.0 * c.T + 4.0 * float((lens * np.diff(row_ptr)).sum())
            + K * 2.0 * staged_rows + 6.0 * float(in_runs.sum()))
    assert model.sampler_bytes()[-1] == want
    model.close()


def test_device_side_argument_errors(mlda):
    import torch
    lib = mlda.load_library()
    c = corpus_synth.tiny(D=10, V=20, K=4, mean_len=5, seed=1)
    model = mlda.Mlda(c.doc_ptr, c.word_ids, 20, 4, 0.5, 0.01, 1)
    with pytest.raises(mlda.MldaError) as e:           # no state yet
        model.step(1)
    assert e.value.code == -1
    with pytest.raises(mlda.MldaError):
        model.assignments()
    with pytest.raises(mlda.MldaError):                # topic >= K
        model.set_assignments(np.full(c.T, 4, dtype=np.uint16))
    model.init_random()
    with pytest.raises(mlda.MldaError):
        model.step(-1)
    model.close()
    bad_words = c.word_ids.copy(); bad_words[3] = 20
    with pytest.raises(mlda.MldaError) as e:
        mlda.Mlda(c.doc_ptr, bad_words, 20, 4, 0.5, 0.01, 1)
    assert e.value.code == -1 and "word id" in str(e.value)
    # host memory handed in as the device workspace
    ctx = ctypes.c_void_p()
    host = np.zeros(1 << 22, dtype=np.uint8)
    addr = (host.ctypes.data + 255) // 256 * 256
    rc = lib.mlda_create(ctypes.addressof(ctx), c.doc_ptr.ctypes.data, c.word_ids.ctypes.data,
                         10, 20, 4, 0.5, 0.01, 1, ctypes.c_void_p(addr), (1 << 22) - 256, None)
    assert rc == -1 and b"not device memory" in lib.mlda_last_error()
    # every K up to 65,535 is served
    big_k = 60000
    model = mlda.Mlda(c.doc_ptr, c.word_ids, 20, big_k, 0.5, 0.01, 1)
    model.close()
