"""The docword (UCI bag-of-words) reader and writer, and the training loop around the library."""
import gzip

import numpy as np
import pytest

import corpus_synth
from paper_1803_04631_amd import bow


def bags(doc_ptr, word_ids):
    return [np.sort(word_ids[doc_ptr[d]:doc_ptr[d + 1]]) for d in range(len(doc_ptr) - 1)]


@pytest.mark.parametrize("suffix", [".txt", ".txt.gz"])
def test_docword_round_trip(tmp_path, suffix):
    c = corpus_synth.tiny(D=40, V=25, K=4, mean_len=9, seed=5)
    lens = np.diff(c.doc_ptr)
    lens[[3, 17, 39]] = 0                                   # some empty documents, the last one too
    keep = np.concatenate([np.arange(c.doc_ptr[d], c.doc_ptr[d] + lens[d]) for d in range(40)])
    doc_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    words = c.word_ids[keep]
    path = tmp_path / ("docword.tiny" + suffix)
    bow.save_docword(path, doc_ptr, words, 25)
    got_ptr, got_words, V = bow.load_docword(path, chunk_lines=37)      # several chunks
    assert V == 25 and np.array_equal(got_ptr, doc_ptr) and got_words.dtype == np.int32
    for a, b in zip(bags(doc_ptr, words), bags(got_ptr, got_words)):
        assert np.array_equal(a, b)
    # inside a document the file order is kept: words ascending, equal words together
    for d in range(40):
        assert np.all(np.diff(got_words[got_ptr[d]:got_ptr[d + 1]]) >= 0)


def test_docword_header_and_lines_are_checked(tmp_path):
    def write(text):
        p = tmp_path / "bad.txt"
        p.write_text(text)
        return p
    good = "2\n3\n3\n1 1 2\n1 3 1\n2 2 4\n"
    ptr, words, V = bow.load_docword(write(good))
    assert V == 3 and ptr.tolist() == [0, 3, 7] and words.tolist() == [0, 0, 2, 1, 1, 1, 1]
    for bad in ("2\n3\n4\n1 1 2\n1 3 1\n2 2 4\n",          # fewer lines than promised
                "2\n3\n3\n1 1 2\n1 4 1\n2 2 4\n",          # word id beyond W
                "2\n3\n3\n1 1 2\n3 3 1\n2 2 4\n",          # document id beyond D
                "2\n3\n3\n2 1 2\n1 3 1\n2 2 4\n",          # not sorted by document
                "2\n3\n3\n1 1 0\n1 3 1\n2 2 4\n"):         # zero count
        with pytest.raises(ValueError):
            bow.load_docword(write(bad))
    with gzip.open(tmp_path / "e.txt.gz", "wt") as f:
        f.write("3\n5\n0\n")
    ptr, words, V = bow.load_docword(tmp_path / "e.txt.gz")
    assert ptr.tolist() == [0, 0, 0, 0] and len(words) == 0 and V == 5


@pytest.mark.gpu
def test_training_from_a_docword_file_raises_the_likelihood(tmp_path):
    import io
    import oracle
    import paper_1803_04631_amd as mlda
    c = corpus_synth.tiny(D=300, V=200, K=10, mean_len=40, seed=9)
    path = tmp_path / "docword.synth.txt.gz"
    bow.save_docword(path, c.doc_ptr, c.word_ids, 200)
    doc_ptr, words, V = bow.load_docword(path)
    log = io.StringIO()
    rows = bow.train(doc_ptr, words, V, K=10, iters=12, every=4, out=log)
    assert [r[0] for r in rows] == [0, 4, 8, 12]
    assert rows[-1][2] > rows[1][2] > rows[0][2]                     # Section 7.2: it rises
    assert all(b[1] >= a[1] for a, b in zip(rows, rows[1:]))
    assert len(log.getvalue().splitlines()) == 5
    # the same twelve iterations through the library directly, and the oracle's likelihood of that state
    m = mlda.Mlda(doc_ptr, words, V, 10, 5.0, 0.01, 4631)
    m.init_random(); m.step(12)
    z = m.assignments()
    n_wk, n_k = oracle.count_word_topic(words, z, V, 10)
    ll = oracle.loglik(doc_ptr, z, V, 10, 5.0, 0.01, n_wk, n_k)
    assert abs(rows[-1][2] * len(words) - ll) <= 1e-5 * abs(ll)
    m.close()
