"""Batches of sentences of different lengths for tv_verify_padded / tv_certify_padded (host logic only).

The kernels take one padded length L per call and compute every padded token, so a batch should hold sentences of
similar length: sentences are sorted by length and cut into batches whose padded length (the longest sentence,
rounded up to the multiple of 4 the kernels need) wastes as little as the batch size allows.
"""
import numpy as np


def padded_length(n, multiple=4):
    return -(-int(n) // multiple) * multiple


def bucket_by_length(lengths, max_batch, multiple=4):
    """Indices of the sentences of each batch and its padded length: [(index array, L), ...].

    Sentences are taken in order of length (stable), a batch is closed when it holds max_batch sentences or when
    the next sentence would raise its padded length."""
    lengths = np.asarray(lengths, dtype=np.int64)
    if lengths.ndim != 1 or len(lengths) == 0 or lengths.min() < 1:
        raise ValueError("lengths must be a non-empty vector of positive integers")
    if max_batch < 1:
        raise ValueError("max_batch must be positive")
    order = np.argsort(lengths, kind="stable")
    batches, cur, cur_L = [], [], None
    for i in order:
        L = padded_length(lengths[i], multiple)
        if cur and (len(cur) == max_batch or L != cur_L):
            batches.append((np.array(cur), cur_L))
            cur = []
        cur.append(int(i))
        cur_L = L
    batches.append((np.array(cur), cur_L))
    return batches


def pad_batch(sentences, idx, L, pad_token=0):
    """tokens [len(idx), L] int32 (rows padded with pad_token) and lengths [len(idx)] int32."""
    tok = np.full((len(idx), L), pad_token, dtype=np.int32)
    lens = np.empty(len(idx), dtype=np.int32)
    for r, i in enumerate(idx):
        s = np.asarray(sentences[i], dtype=np.int32)
        if s.ndim != 1 or len(s) > L:
            raise ValueError(f"sentence {i} does not fit the padded length {L}")
        tok[r, :len(s)] = s
        lens[r] = len(s)
    return tok, lens
