"""Page contents: every 8-byte word of every page is a fixed function of
(page id, word index), so any copy of a page can be checked wherever it lives.

The mixing function is the public-domain SplitMix64 output stage applied to an
affine combination of the two counters.  A numpy and a torch implementation
are given; the torch one runs on the device so multi-GiB backing stores can be
filled and verified without a host loop.
"""
import numpy as np

_M = (1 << 64) - 1
_A = 0x9E3779B97F4A7C15
_B = 0xBF58476D1CE4E5B9
_C = 0x94D049BB133111EB


def mix64(p, k):
    """uint64 hash of counters (p, k); accepts python ints or numpy arrays."""
    with np.errstate(over="ignore"):
        p = np.asarray(p, dtype=np.uint64)
        k = np.asarray(k, dtype=np.uint64)
        z = p * np.uint64(_A) + k * np.uint64(_B) + np.uint64(_C)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_B)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_C)
        return z ^ (z >> np.uint64(31))


def page_words(pages, words_per_page):
    """Initial contents of `pages` as uint64 [len(pages), words_per_page]."""
    pages = np.asarray(pages, dtype=np.uint64).reshape(-1, 1)
    k = np.arange(words_per_page, dtype=np.uint64).reshape(1, -1)
    return mix64(pages, k)


STAMP_TAG = 1 << 32


def stamp_of(pages, epoch, words_per_page):
    """A write the running task makes to each of `pages` during scheduling
    epoch `epoch`: returns (word index, value) per page.  Word index and value
    both depend on (page, epoch), so successive writes land on different words."""
    pages = np.asarray(pages, dtype=np.uint64)
    h = mix64(pages, np.uint64(STAMP_TAG + epoch))
    idx = (h % np.uint64(words_per_page)).astype(np.int64)
    val = mix64(h, pages)
    return idx, val


# ---- torch twin (device-side fill / verify) ------------------------------------

def _t_const(x):
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(z, s):
    # logical shift right of an int64 tensor
    return (z >> s) & ((1 << (64 - s)) - 1)


def mix64_torch(p, k):
    """Same function on int64 torch tensors (bit pattern of the uint64 result)."""
    z = p * _t_const(_A) + k * _t_const(_B) + _t_const(_C)
    z = (z ^ _lsr(z, 30)) * _t_const(_B)
    z = (z ^ _lsr(z, 27)) * _t_const(_C)
    return z ^ _lsr(z, 31)


def page_words_torch(pages, words_per_page):
    """int64 [n, words_per_page] on the device of `pages` (an int64 tensor)."""
    import torch
    k = torch.arange(words_per_page, dtype=torch.int64, device=pages.device).reshape(1, -1)
    return mix64_torch(pages.reshape(-1, 1), k)
