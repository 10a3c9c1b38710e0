"""What every correct layout of routed rows has in common, whatever the order inside a region.

Counts, offsets and the per-destination view are unique; the slot maps are only required to be
inverse bijections that put every flat row inside the region of its expert (dense packing,
nothing dropped).  Plain numpy; used for the arrival-order layouts, whose row order is not unique.
"""
import numpy as np


def check_layout_is_valid(topk_idx, E, G, lay):
    flat = np.asarray(topk_idx, np.int64).ravel()
    R = flat.size
    cnt = np.bincount(flat, minlength=E)
    off = np.concatenate([[0], np.cumsum(cnt)])
    Eg = E // G
    assert np.array_equal(lay["expert_counts"], cnt), "expert_counts"
    assert np.array_equal(lay["expert_offsets"], off), "expert_offsets"
    assert np.array_equal(lay["dest_counts"], cnt.reshape(G, Eg).sum(axis=1)), "dest_counts"
    assert np.array_equal(lay["dest_offsets"], off[0:E + 1:Eg]), "dest_offsets"
    slot = np.asarray(lay["slot_of_row"], np.int64)
    row = np.asarray(lay["row_of_slot"], np.int64)
    assert slot.shape == (R,) and row.shape == (R,)
    if R == 0:
        return
    assert slot.min() >= 0 and slot.max() < R and row.min() >= 0 and row.max() < R, "range"
    assert np.array_equal(np.sort(slot), np.arange(R)), "slot_of_row is not a bijection"
    assert np.array_equal(row[slot], np.arange(R)), "row_of_slot is not the inverse of slot_of_row"
    assert np.all(slot >= off[flat]) and np.all(slot < off[flat + 1]), "row outside its expert's region"
