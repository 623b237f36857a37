"""Reference for the segment table: token rows grouped by adapter.

The grouping is a stable sort of the rows by adapter id (ascending, rows with
no adapter last), which is unique; a library stable sort is the definition
written out.  TEST INFRASTRUCTURE ONLY."""
from __future__ import annotations

import numpy as np


def plan_reference(req_adapter, req_ntok, ranks):
    req_adapter = np.asarray(req_adapter, np.int64)
    req_ntok = np.asarray(req_ntok, np.int64)
    ranks = np.asarray(ranks, np.int64)
    n_ad = ranks.shape[0]
    row_ad = np.repeat(req_adapter, req_ntok)
    key = np.where(row_ad < 0, n_ad, row_ad)
    perm = np.argsort(key, kind="stable").astype(np.int32)
    skey = key[perm]
    seg_key, seg_start = np.unique(skey, return_index=True)
    seg_indptr = np.concatenate([seg_start, [skey.shape[0]]]).astype(np.int32)
    seg_adapter = np.where(seg_key == n_ad, -1, seg_key).astype(np.int32)
    seg_rank = np.where(seg_adapter >= 0, ranks[np.maximum(seg_adapter, 0)] if n_ad else 0, 0).astype(np.int32)
    seg_ext = np.concatenate([[0], np.cumsum(seg_rank)]).astype(np.int32)
    row_seg = (np.searchsorted(seg_indptr, np.arange(skey.shape[0]), side="right") - 1).astype(np.int32)
    return dict(perm=perm, seg_adapter=seg_adapter, seg_indptr=seg_indptr, seg_rank=seg_rank,
                seg_ext=seg_ext, row_seg=row_seg, n_seg=int(seg_adapter.shape[0]))
