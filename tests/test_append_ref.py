"""The plain-Python statement of the KV append, checked against what it must do by construction."""
import numpy as np

from oracle import append_ref
from paper_2604_23838_amd import workloads as W


def test_append_ref_writes_exactly_one_slot_per_active_request():
    shp = W.SHAPES[1]
    w = W.build(shp, [31, 5, 0, 16], seed=1, cfg=98, poison=False)
    bt = w.block_table.copy()
    assert bt.shape[1] == 2
    free = sorted(set(range(w.num_pages)) - set(bt[bt >= 0].tolist()))
    bt[3, 1] = free[0]                            # request 3 sits on a page boundary: its next page is assigned
    bt[2, 0] = free[1]                            # request 2 is an empty slot with a page ready for its first token
    rng = np.random.default_rng(0)
    kn = W.f32_to_bf16_bits(rng.standard_normal((4, 2, 64), dtype=np.float32))
    vn = W.f32_to_bf16_bits(rng.standard_normal((4, 2, 64), dtype=np.float32))
    k2, v2, l2 = append_ref.append_kv(kn, vn, w.k_pages, w.v_pages, bt, w.seq_lens)
    assert l2.tolist() == [32, 6, 0, 17]          # the empty slot is not a running request
    changed = np.argwhere((k2 != w.k_pages).any(axis=3))
    want = {(int(bt[0, 1]), 15), (int(bt[1, 0]), 5), (int(bt[3, 1]), 0)}
    assert {(int(p), int(s)) for p, _, s in changed} == want
    for b, (pg, slot) in zip((0, 1, 3), ((int(bt[0, 1]), 15), (int(bt[1, 0]), 5), (int(bt[3, 1]), 0))):
        assert np.array_equal(k2[pg, :, slot, :], kn[b]) and np.array_equal(v2[pg, :, slot, :], vn[b])
    # inputs are not modified; an explicit mask overrides the L > 0 rule; a full request is left alone
    assert w.seq_lens.tolist() == [31, 5, 0, 16]
    k3, v3, l3 = append_ref.append_kv(kn, vn, k2, v2, bt, l2, active=[1, 0, 1, 0])
    assert l3.tolist() == [32, 6, 1, 17]          # request 0 is at capacity (2 pages), request 2 starts
    assert np.array_equal(k3[free[1], :, 0, :], kn[2])
    bt[2, 0] = -1                                 # without an assigned page the request is left alone
    assert append_ref.append_kv(kn, vn, k2, v2, bt, l2, active=[0, 0, 1, 0])[2].tolist() == [32, 6, 0, 17]
