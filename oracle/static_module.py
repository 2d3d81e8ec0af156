"""CPU ORACLE of the cache's static module -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Paper Section 4.2: scan the dataset (or a sample of it), count how often every id occurs, and re-order the
embedding rows "from high to low according to occurrence frequency"; idx_map converts an id to its row in the
re-ordered table.  Plain numpy, straight from that definition; ids with equal counts keep ascending id order
(the paper does not say; a stable order is needed for a unique answer).
Pinned in tests/test_oracle_pins.py by a hand example, by Python's own sort on (-count, id) tuples, and by the
properties that define the result.
"""
import numpy as np


def count_ids(batches, num_rows: int) -> np.ndarray:
    """Occurrences of every id over an iterable of int64 id arrays."""
    counts = np.zeros(num_rows, dtype=np.int64)
    for ids in batches:
        ids = np.asarray(ids)
        if ids.size and (ids.min() < 0 or ids.max() >= num_rows):
            raise ValueError("id out of range")
        np.add.at(counts, ids, 1)
    return counts


def freq_rank_from_counts(counts: np.ndarray):
    """(freq_rank, inv_rank): inv_rank lists ids by descending count, ties by ascending id; freq_rank inverts it."""
    n = counts.shape[0]
    inv_rank = np.argsort(-counts.astype(np.int64), kind="stable").astype(np.int32)
    freq_rank = np.empty(n, dtype=np.int32)
    freq_rank[inv_rank] = np.arange(n, dtype=np.int32)
    return freq_rank, inv_rank


def reorder_table(table: np.ndarray, inv_rank: np.ndarray) -> np.ndarray:
    """Row r of the result is the embedding of the id with frequency rank r."""
    return table[inv_rank]
