"""Bag-of-words corpora in the UCI `docword` text format, and a training loop that prints the
log-likelihood per token against time (the paper's Section 7.1 names the format's two
collections, NYTimes and PubMed; Section 7.2 plots log-likelihood per token over time).

Format: three header lines D, W, NNZ, then NNZ lines `docID wordID count` with 1-based ids,
sorted by document.  A corpus file may be gzip-compressed.  The files themselves are not
part of this repository.

    python -m paper_1803_04631_amd.bow docword.nytimes.txt.gz --topics 1000 --iters 100
"""
from __future__ import annotations

import argparse
import gzip
import sys
import time

import numpy as np


def _open(path, mode):
    return gzip.open(path, mode) if str(path).endswith(".gz") else open(path, mode)


def load_docword(path, chunk_lines: int = 1 << 22):
    """Read a docword file.  Returns (doc_ptr int64[D+1], word_ids int32[T], V): every
    (document, word, count) line becomes `count` consecutive tokens of that word, documents in
    file order; documents without lines are empty."""
    import pandas as pd
    with _open(path, "rt") as f:
        D, V, nnz = (int(f.readline()) for _ in range(3))
        lengths = np.zeros(D, dtype=np.int64)
        words, seen, last_doc = [], 0, 0
        reader = pd.read_csv(f, sep=r"\s+", header=None, names=["d", "w", "c"], dtype=np.int64,
                             chunksize=chunk_lines, engine="c")
        for part in reader:
            d, w, c = part["d"].to_numpy(), part["w"].to_numpy(), part["c"].to_numpy()
            if len(d) == 0:
                continue
            if d.min() < 1 or d.max() > D or w.min() < 1 or w.max() > V or c.min() < 1:
                raise ValueError("docword: id or count out of range")
            if d[0] < last_doc or np.any(np.diff(d) < 0):
                raise ValueError("docword: lines must be sorted by document")
            last_doc = int(d[-1])
            np.add.at(lengths, d - 1, c)
            words.append(np.repeat((w - 1).astype(np.int32), c))
            seen += len(d)
    if seen != nnz:
        raise ValueError(f"docword: header promises {nnz} lines, file has {seen}")
    doc_ptr = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    word_ids = np.concatenate(words) if words else np.zeros(0, dtype=np.int32)
    return doc_ptr, word_ids, V


def save_docword(path, doc_ptr, word_ids, V: int):
    """Write a corpus in the docword format (one line per distinct word of a document)."""
    doc_ptr = np.asarray(doc_ptr, dtype=np.int64)
    word_ids = np.asarray(word_ids, dtype=np.int64)
    D = len(doc_ptr) - 1
    doc_of = np.repeat(np.arange(D, dtype=np.int64), np.diff(doc_ptr))
    pairs, counts = np.unique(doc_of * V + word_ids, return_counts=True)
    with _open(path, "wt") as f:
        f.write(f"{D}\n{V}\n{len(pairs)}\n")
        np.savetxt(f, np.column_stack([pairs // V + 1, pairs % V + 1, counts]), fmt="%d")


def train(doc_ptr, word_ids, V: int, K: int, iters: int, seed: int = 4631, every: int = 1,
          chunks: int = 1, out=sys.stdout):
    """Run `iters` iterations with alpha = 50/K, beta = 0.01 (Section 7) from random topics and
    print iteration, seconds since the start of sampling and log-likelihood per token.
    Returns the rows as a list of (iteration, seconds, loglik_per_token)."""
    import torch
    from . import Mlda
    T = len(word_ids)
    model = Mlda(doc_ptr, word_ids, V, K, 50.0 / K, 0.01, seed, chunks=chunks)
    model.init_random()
    rows = [(0, 0.0, model.loglik() / max(T, 1))]
    print("iteration seconds loglik_per_token", file=out)
    print("%d %.3f %.6f" % rows[0], file=out, flush=True)
    torch.cuda.synchronize()
    spent = 0.0
    done = 0
    while done < iters:
        n = min(every, iters - done)
        t0 = time.perf_counter()
        model.step(n, loglik=False)
        model.synchronize()
        torch.cuda.synchronize()
        spent += time.perf_counter() - t0          # the likelihood is not part of the training time
        done += n
        rows.append((done, spent, model.loglik() / max(T, 1)))
        print("%d %.3f %.6f" % rows[-1], file=out, flush=True)
    model.close()
    return rows


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("docword", help="docword.*.txt or .txt.gz")
    ap.add_argument("--topics", type=int, default=1000)
    ap.add_argument("--iters", type=int, default=100)
    ap.add_argument("--every", type=int, default=5, help="iterations between likelihood evaluations")
    ap.add_argument("--chunks", type=int, default=1, help="stream the corpus through the GPU in chunks")
    ap.add_argument("--seed", type=int, default=4631)
    args = ap.parse_args(argv)
    t0 = time.perf_counter()
    doc_ptr, word_ids, V = load_docword(args.docword)
    print("# %d documents, %d words, %d tokens, read in %.1f s"
          % (len(doc_ptr) - 1, V, len(word_ids), time.perf_counter() - t0), file=sys.stderr)
    train(doc_ptr, word_ids, V, args.topics, args.iters, seed=args.seed, every=args.every,
          chunks=args.chunks)


if __name__ == "__main__":
    main()
