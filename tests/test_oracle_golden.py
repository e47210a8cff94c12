"""The oracle against the hand-worked fixture in tests/golden/hand_worked_two_tables.txt."""
import os

import numpy as np


def _load():
    d = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_two_tables.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split(":")
        d[k.strip()] = [float(x) for x in v.split()]
    return d


def test_hand_worked_example(ora):
    g = _load()
    i32 = lambda k: np.array(g[k], dtype=np.int32)
    rows = [int(x) for x in g["rows"]]
    D, B = int(g["D"][0]), int(g["B"][0])
    tabs = lambda: [np.array(g["table0"], dtype=np.float32).reshape(-1, D),
                    np.array(g["table1"], dtype=np.float32).reshape(-1, D)]
    idx, off = i32("indices"), i32("offsets")
    rc, counts = ora.histogram(rows, idx, off, B)
    assert rc == 0 and counts.tolist() == g["counts"]
    k = ora.budget_rows(sum(rows), int(g["row_bytes"][0]), int(g["budget_bytes"][0]))
    assert k == g["k"][0]
    rc, hot, slot_of = ora.hot_set(counts, k)
    assert hot.tolist() == g["hot_gid"] and slot_of.tolist() == g["slot_of"]
    rc, slot, hit, miss, mg = ora.remap(rows, idx, off, B, slot_of)
    assert slot.tolist() == g["slot"] and hit.tolist() == g["hit_pos"]
    assert miss.tolist() == g["miss_pos"] and mg.tolist() == g["miss_gid"]
    rc, out = ora.embedding_bag_fwd(rows, tabs(), idx, off, B)
    assert out.reshape(-1).tolist() == g["out"]
    allrows = np.concatenate(tabs())
    rc, out2 = ora.embedding_bag_fwd(rows, tabs(), idx, off, B, slot_of, np.ascontiguousarray(allrows[hot]))
    assert out2.reshape(-1).tolist() == g["out"]
    rc, sg, sb, ss, ug = ora.bwd_segments(rows, idx, off, B)
    assert sg.tolist() == g["sorted_gid"] and sb.tolist() == g["sorted_bag"]
    assert ss.tolist() == g["seg_start"] and ug.tolist() == g["unique_gid"]
    grad = np.array(g["grad_out"], dtype=np.float32).reshape(-1, D)
    t = tabs()
    rc, nr, ns, gr = ora.embedding_bag_bwd_update(rows, t, None, 0, idx, off, B, grad, g["sgd_lr"][0], 0.0,
                                                  report=True, n_unique=ug.size)
    assert gr.reshape(-1).tolist() == g["grad_rows"]
    ora.embedding_bag_bwd_update(rows, t, None, 0, idx, off, B, grad, g["sgd_lr"][0], 0.0)
    assert np.concatenate(t).reshape(-1).tolist() == g["sgd_rows"]
    t = tabs()
    st = [np.zeros_like(x) for x in t]
    ora.embedding_bag_bwd_update(rows, t, st, 1, idx, off, B, grad, g["adagrad_lr"][0], g["adagrad_eps"][0])
    assert np.concatenate(st).reshape(-1).tolist() == g["adagrad_state"]
    np.testing.assert_allclose(np.concatenate(t).reshape(-1), np.array(g["adagrad_rows"]), rtol=1e-7, atol=0)
