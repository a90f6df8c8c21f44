"""Helpers for the GPU parity tests: oracle-side expectations for device tables."""
from __future__ import annotations

import numpy as np
import torch


def bits_from_table(rows: np.ndarray, row_words: int) -> np.ndarray:
    """Allowed-bit rows (uint32 words, bit t&31 of word t>>5) that a table's rows imply."""
    n, v = rows.shape
    live = np.zeros((n, row_words * 32), dtype=np.uint8)
    live[:, :v] = rows >= 0
    return np.packbits(live, axis=1, bitorder="little").view(np.uint32).reshape(n, row_words)


def check_rows(table, oracle_rows: np.ndarray, row_ids) -> None:
    """Device rows `row_ids` of delta and allow equal the oracle's rows, bit for bit."""
    idx = torch.as_tensor(np.asarray(row_ids), device=table.delta.device, dtype=torch.long)
    got = table.delta.index_select(0, idx).cpu().numpy()
    assert got.dtype == np.int32 and got.shape == oracle_rows.shape
    if not np.array_equal(got, oracle_rows):
        bad = np.argwhere(got != oracle_rows)
        r, c = bad[0]
        raise AssertionError(f"{len(bad)} table entries differ; first at row {row_ids[r]} token {c}: "
                             f"gpu {got[r, c]} oracle {oracle_rows[r, c]}")
    bits = table.allow.index_select(0, idx).cpu().numpy().view(np.uint32)
    want = bits_from_table(oracle_rows, table.row_words)
    assert np.array_equal(bits, want), "allowed-bit rows differ"
