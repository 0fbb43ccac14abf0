"""CPU-only checks of the library boundary and its host-side integer bookkeeping:
the shared library loads and exports every function the header declares, the transposed index is
the exact transpose, packed index words decode to (vertex, chunk), the launch schedule partitions
the entries, and descriptor validation reports errors without touching a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from synth import graphs
from synth.configs import CONFIGS, make_graph

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    import paper_2308_10087_amd as g
    return g


def test_library_exports_every_declared_symbol():
    g = _lib()
    import glob
    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert [os.path.basename(h) for h in headers] == ["gnnstage.h", "gnntrain.h"]
    header = "\n".join(open(h).read() for h in headers)
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = re.findall(r"\b([a-z_][a-z0-9_]*)\s*\(", header)
    declared = sorted({n for n in names if n.startswith(("gnnstage_", "gnntrain_", "stage_", "update_history"))})
    assert {"gnnstage_create", "stage_forward_chunk", "stage_backward_chunk", "update_history",
            "gnnstage_destroy", "gnntrain_create", "gnntrain_epoch", "gnntrain_chunk_order", "gnntrain_softmax_xent",
            "gnntrain_adam_step", "gnntrain_sgd_step", "gnntrain_sum", "gnnstage_query", "gnnstage_buffer",
            "gnnstage_partition_chunks", "gnnstage_permute_csr", "gnnstage_set_dropout_seed",
            "gnnstage_set_dropout_rate"} <= set(declared)
    for name in declared:
        assert hasattr(g.lib, name), name
    assert g.gnnstage_version() >= 100


def test_dense_block_launcher_refuses_a_launch_with_a_missing_operand():
    """The dense-block kernel reads all of its operand tables without a test of its own (a null table is a memory
    fault on the device), so the launcher must refuse - on the host, before anything is launched."""
    g = _lib()
    g.lib.gnnstage_debug_dense_rejects.restype = C.c_int
    g.lib.gnnstage_debug_dense_rejects.argtypes = [C.c_int32, C.c_int32]
    for pattern in (0, 1):
        for missing in range(6 if pattern else 5):
            assert g.lib.gnnstage_debug_dense_rejects(missing, pattern) == 1, (missing, pattern)
    assert g.lib.gnnstage_debug_dense_rejects(5, 0) == -1 and g.lib.gnnstage_debug_dense_rejects(9, 1) == -1


def test_chunk_order_matches_the_oracle_bit_for_bit():
    """Section 3.4, technique 1: the library's host-side shuffle and the oracle's draw the same orders."""
    from oracle.train import chunk_order
    g = _lib()
    for seed in (0, 1, 2308100900, (1 << 64) - 1, 0x9E3779B97F4A7C15):
        for K in (1, 2, 7, 8, 32, 256):
            for epoch in (0, 1, 2, 77, 10**6):
                assert np.array_equal(g.gnntrain_chunk_order(seed, epoch, K), chunk_order(seed, epoch, K)), (seed, K, epoch)
    assert np.array_equal(g.gnntrain_chunk_order(5, 3, 9, shuffle=False), np.arange(9))


def test_chunk_partitioner_matches_the_oracle_bit_for_bit():
    """Algorithm 1's first step on the host: the library's restreaming-FENNEL partitioner and the oracle's make the
    same decision for every vertex (integer parts; the scores are plain IEEE operations on both sides)."""
    from oracle.partition import edge_cut, partition_chunks, permute_csr
    from synth.configs import CONFIGS, make_graph
    g = _lib()
    cases = [
        (graphs.planted_partition(3000, 8, 10.0, 2.0, 3)[:2], 8, dict()),
        (graphs.erdos_renyi(1500, 7.0, 4), 5, dict(passes=2, slack=1.05, balance=1.0)),
        (make_graph(CONFIGS["c1_s"]), 8, dict(passes=3)),
        (make_graph(CONFIGS["c3_s"]), 16, dict(passes=4, slack=1.3)),
        (graphs.erdos_renyi(200, 4.0, 5), 1, dict()),
        (graphs.erdos_renyi(97, 3.0, 6), 97, dict(passes=2, slack=1.0)),    # one vertex per chunk
        (make_graph(CONFIGS["c1_s"]), 8, dict(by_entries=True)),
        (make_graph(CONFIGS["c2_s"]), 16, dict(by_entries=True, passes=3, slack=1.05, balance=2.0)),
    ]
    for (row_ptr, col), K, kw in cases:
        part, perm, chunk_ptr = g.gnnstage_partition_chunks(row_ptr, col, K, **kw)
        okw = dict(kw)
        if "slack" in okw:
            okw["nu"] = okw.pop("slack")
        rpart, rperm, rchunk = partition_chunks(row_ptr, col, K, **okw)
        assert np.array_equal(part, rpart) and np.array_equal(perm, rperm) and np.array_equal(chunk_ptr, rchunk), K
        p2, c2 = g.gnnstage_permute_csr(row_ptr, col, perm)
        q2, d2 = permute_csr(row_ptr, col, perm)
        assert np.array_equal(p2, q2) and np.array_equal(c2, d2)
    # what it is for: far fewer neighbours in other chunks than index ranges of randomly numbered vertices
    (row_ptr, col), K, _ = cases[0]
    part, perm, chunk_ptr = g.gnnstage_partition_chunks(row_ptr, col, K)
    blind = (np.arange(3000) * K // 3000).astype(np.int32)
    assert edge_cut(row_ptr, col, part) < 0.3 * edge_cut(row_ptr, col, blind)
    with pytest.raises(g.GnnStageError):
        g.gnnstage_permute_csr(row_ptr, col, np.zeros(3000, dtype=np.int32))     # not a permutation
    empty = np.zeros(8, dtype=np.int64)                 # seven vertices, no entries: nothing to balance by entries
    none = np.zeros(0, dtype=np.int32)
    with pytest.raises(g.GnnStageError):
        g.gnnstage_partition_chunks(empty, none, 2, by_entries=True)
    with pytest.raises(ValueError):
        partition_chunks(empty, none, 2, by_entries=True)
    part, perm, chunk_ptr = g.gnnstage_partition_chunks(empty, none, 9)          # more chunks than vertices
    rpart, rperm, rchunk = partition_chunks(empty, none, 9)
    assert np.array_equal(part, rpart) and np.array_equal(perm, rperm) and np.array_equal(chunk_ptr, rchunk)
    assert chunk_ptr[-1] == 7 and sorted(perm.tolist()) == list(range(7))


def test_transposed_index_is_the_exact_transpose():
    g = _lib()
    rng = np.random.default_rng(1)
    n = 300
    row_ptr, col = graphs.from_directed_pairs(n, rng.integers(0, n, 4000), rng.integers(0, n, 4000))
    t_ptr, t_row, t_edge = g.gnnstage_plan_transpose(row_ptr, col)
    # same as the oracle's own transposition (independent code)
    st = oracle.OracleStage(row_ptr, col, np.ones(len(col), np.float32), [0, n], [1, 1], [np.ones((1, 1), np.float32)])
    assert np.array_equal(t_ptr, st.t_ptr) and np.array_equal(t_row, st.t_row) and np.array_equal(t_edge, st.t_edge)
    # transposing the transpose gives the CSR back
    b_ptr, b_row, _ = g.gnnstage_plan_transpose(t_ptr, t_row)
    assert np.array_equal(b_ptr, row_ptr) and np.array_equal(b_row, col)
    # every entry points back at itself
    rows_of_edge = np.repeat(np.arange(n), np.diff(row_ptr))
    assert np.array_equal(rows_of_edge[t_edge], t_row)
    assert np.array_equal(col[t_edge], np.repeat(np.arange(n), np.diff(t_ptr)))
    with pytest.raises(g.GnnStageError):
        g.gnnstage_plan_transpose(np.array([0, 1]), np.array([5]))  # column out of range


@pytest.mark.parametrize("n,k", [(1000, 7), (5, 1), (70000, 200)])
def test_packed_words_decode_to_vertex_and_chunk(n, k):
    g = _lib()
    rng = np.random.default_rng(2)
    idx = rng.integers(0, n, 5000).astype(np.int32)
    chunk_ptr = graphs.ragged_chunks(n, k, 3) if k > 1 else np.array([0, n])
    packed, vbits = g.gnnstage_plan_pack(n, idx, chunk_ptr)
    assert (1 << vbits) >= n
    assert np.array_equal(packed & ((1 << vbits) - 1), idx.astype(np.uint32))
    want_chunk = np.searchsorted(chunk_ptr, idx, side="right") - 1
    assert np.array_equal(packed >> vbits, want_chunk.astype(np.uint32))


def test_packing_refuses_sizes_beyond_32_bits():
    g = _lib()
    vb = C.c_int32(0)
    cp = np.array([0] + [1 << 27] * 255 + [1 << 28], dtype=np.int64)
    rc = g.lib.gnnstage_plan_pack(1 << 28, 0, None, 256, cp.ctypes.data, None, C.byref(vb))
    assert rc == -6  # 28 vertex bits + 8 chunk bits > 32


@pytest.mark.parametrize("split,classes", [(64, 1), (500, 1), (1 << 20, 1), (64, 8), (300, 8), (1 << 20, 3)])
def test_launch_schedule_partitions_the_entries(split, classes):
    g = _lib()
    w = CONFIGS["c4_s"]
    row_ptr, col = make_graph(w)
    n = len(row_ptr) - 1
    chunk_ptr = graphs.equal_chunks(n, 5)
    covered = np.zeros(row_ptr[-1], dtype=np.int32)
    min_row = 100
    for c in range(5):
        row, e0, ne, slot, n_slots, class_off, slot_class = g.gnnstage_plan_tasks(
            row_ptr, int(chunk_ptr[c]), int(chunk_ptr[c + 1]), split, idx=col, n_vertices=n, n_classes=classes,
            class_min_row=min_row, return_classes=True)
        assert np.all(ne <= split) and np.all(ne >= 0)
        assert np.all((row >= chunk_ptr[c]) & (row < chunk_ptr[c + 1]))
        for r, a, m in zip(row, e0, ne):
            assert row_ptr[r] <= a and a + m <= row_ptr[r + 1]
            covered[a:a + m] += 1
        deg = np.diff(row_ptr)[chunk_ptr[c]:chunk_ptr[c + 1]]
        is_cut = (deg > split) | ((classes > 1) & (deg >= min_row))
        cut_rows = np.flatnonzero(is_cut) + chunk_ptr[c]
        # whole rows carry slot -1 and appear once, after every piece of the cut rows
        whole = row[slot < 0]
        assert len(np.unique(whole)) == len(whole) == (~is_cut).sum()
        pieces = np.sort(slot[slot >= 0])
        assert np.array_equal(pieces, np.arange(n_slots))
        assert np.all(slot[:len(pieces)] >= 0)
        assert set(row[slot >= 0].tolist()) == set(cut_rows.tolist())
        # slots of one row are consecutive (the reduce kernel sums slot0 .. slot0 + count - 1)
        order = np.argsort(slot[slot >= 0])
        rows_by_slot = row[slot >= 0][order]
        assert np.all(np.diff(rows_by_slot) >= 0) or len(np.unique(rows_by_slot)) == (np.diff(rows_by_slot) != 0).sum() + 1
        assert np.all(np.diff(class_off) >= 0) and class_off[0] == 0
        if classes > 1:
            # class-major sections: section q holds exactly the pieces that gather from source-id range q
            for q in range(classes):
                for i in range(class_off[q], class_off[q + 1]):
                    cls = col[e0[i]:e0[i] + ne[i]].astype(np.int64) * classes // n
                    assert ne[i] > 0 and cls.min() == cls.max() == q and slot_class[slot[i]] == q
            tail = slice(class_off[classes], len(row))
            assert np.all(slot_class[slot[tail][slot[tail] >= 0]] == 255)
        else:
            assert class_off[classes] == 0 and np.all(slot_class == 255)
    assert np.all(covered == 1)  # every entry belongs to exactly one task


def test_launch_schedule_with_explicit_class_bounds():
    """Class sections follow the given id bounds (here: uneven ones), not equal id ranges."""
    g = _lib()
    w = CONFIGS["c3_s"]
    row_ptr, col = make_graph(w)
    n = len(row_ptr) - 1
    lo = np.array([0, n // 10, n // 2, n // 2 + 7, n], dtype=np.int64)
    row, e0, ne, slot, n_slots, class_off, slot_class = g.gnnstage_plan_tasks(
        row_ptr, 0, n, 128, idx=col, n_vertices=n, n_classes=4, class_min_row=8, return_classes=True, class_lo=lo)
    covered = np.zeros(row_ptr[-1], dtype=np.int32)
    for r, a, m in zip(row, e0, ne):
        covered[a:a + m] += 1
    assert np.all(covered == 1)
    assert class_off[4] > 0
    for q in range(4):
        for i in range(class_off[q], class_off[q + 1]):
            u = col[e0[i]:e0[i] + ne[i]]
            assert ne[i] > 0 and u.min() >= lo[q] and u.max() < lo[q + 1] and slot_class[slot[i]] == q
    with pytest.raises(g.GnnStageError):
        g.gnnstage_plan_tasks(row_ptr, 0, n, 128, idx=col, n_vertices=n, n_classes=4, class_min_row=8,
                              class_lo=np.array([0, 5, 3, 9, n]))  # not ascending


def test_launch_schedule_with_classes_that_end_before_the_last_id():
    """Hotness classes: the index handed to the planner holds, per entry, the RANK of its source (0 = most
    often gathered), ascending inside every row; classes are slices of the first ranks only, and the run of a
    row beyond the last class is cut into pieces without a class."""
    g = _lib()
    w = CONFIGS["c4_s"]
    row_ptr, col = make_graph(w)
    n = len(row_ptr) - 1
    count = np.bincount(col, minlength=n)
    by_hotness = np.lexsort((np.arange(n), -count))          # descending count, ties by id
    rank_of = np.empty(n, dtype=np.int64)
    rank_of[by_hotness] = np.arange(n)
    ranks = rank_of[col]
    for v in range(n):                                        # every row ascending in rank
        ranks[row_ptr[v]:row_ptr[v + 1]].sort()
    ranks = ranks.astype(np.int32)
    R, classes, min_row, split = 40, 4, 16, 64
    lo = np.arange(classes + 1, dtype=np.int64) * R           # ends at rank 160 of 30,011
    row, e0, ne, slot, n_slots, class_off, slot_class = g.gnnstage_plan_tasks(
        row_ptr, 0, n, split, idx=ranks, n_vertices=n, n_classes=classes, class_min_row=min_row, return_classes=True,
        class_lo=lo)
    covered = np.zeros(row_ptr[-1], dtype=np.int32)
    for r, a, m in zip(row, e0, ne):
        assert row_ptr[r] <= a and a + m <= row_ptr[r + 1] and m <= split
        covered[a:a + m] += 1
    assert np.all(covered == 1)
    assert class_off[classes] > 0
    for q in range(classes):
        for i in range(class_off[q], class_off[q + 1]):
            u = ranks[e0[i]:e0[i] + ne[i]]
            assert ne[i] > 0 and u.min() >= lo[q] and u.max() < lo[q + 1] and slot_class[slot[i]] == q
    deg = np.diff(row_ptr)
    n_pieces = int((slot >= 0).sum())
    tail_pieces = [i for i in range(class_off[classes], n_pieces)]
    assert tail_pieces, "some long row must have a run beyond the classes"
    for i in tail_pieces:                                     # class-less pieces: only ranks beyond the classes,
        u = ranks[e0[i]:e0[i] + ne[i]]                        # or rows too short to be cut by class at all
        assert slot_class[slot[i]] == 255
        assert u.min() >= lo[classes] or deg[row[i]] < min_row
    # a long row's sections appear in rank order: its class pieces cover exactly its entries below the last bound
    long_rows = np.flatnonzero(deg >= min_row)
    in_class = np.zeros(row_ptr[-1], dtype=bool)
    for i in range(class_off[classes]):
        in_class[e0[i]:e0[i] + ne[i]] = True
    for v in long_rows[:200]:
        seg = slice(row_ptr[v], row_ptr[v + 1])
        assert np.array_equal(in_class[seg], ranks[seg] < lo[classes])
    with pytest.raises(g.GnnStageError):
        g.gnnstage_plan_tasks(row_ptr, 0, n, split, idx=ranks, n_vertices=n, n_classes=classes, class_min_row=min_row,
                              class_lo=np.array([0, 5, 9, 12, n + 1]))  # beyond the id range


@pytest.mark.parametrize("name,min_nnz", [("c1_s", 40), ("c3_s", 12), ("c0", 3)])
def test_dense_plan_partitions_the_entries(name, min_nnz):
    """Dense blocks + remainder hold every entry exactly once, at the right (row, column); rows and columns
    of a block come from one chunk each; every dense block reaches the threshold."""
    g = _lib()
    w = CONFIGS[name]
    row_ptr, col = make_graph(w)
    n = len(row_ptr) - 1
    chunk_ptr = graphs.ragged_chunks(n, 5, 3)
    d = g.gnnstage_dense_plan(row_ptr, col, chunk_ptr, min_nnz, 0.0)
    assert len(d["blk_rb"]) > 0, "threshold too high for this graph: nothing to check"
    rows_of_entry = np.repeat(np.arange(n), np.diff(row_ptr))
    seen = np.zeros(row_ptr[-1], dtype=np.int32)
    # remainder: same rows, original order, columns unchanged
    seen[d["rem_orig"]] += 1
    assert np.array_equal(d["rem_idx"], col[d["rem_orig"]])
    assert np.array_equal(np.repeat(np.arange(n), np.diff(d["rem_ptr"])), rows_of_entry[d["rem_orig"]])
    assert np.all(np.diff(d["rem_orig"]) > 0)
    # orders are permutations inside every chunk, sorted by length / column frequency
    col_count = np.bincount(col, minlength=n)
    for c in range(5):
        a, b = chunk_ptr[c], chunk_ptr[c + 1]
        rp = d["row_perm"][a:b]
        assert np.array_equal(np.sort(rp), np.arange(a, b))
        assert np.all(np.diff(np.diff(row_ptr)[rp]) <= 0)
        slots = d["colslot_vertex"][d["cb_off"][c] * 64:d["cb_off"][c + 1] * 64]
        real = slots[slots >= 0]
        assert np.array_equal(np.sort(real), np.arange(a, b)) and np.all(slots[len(real):] == -1)
        assert np.all(np.diff(col_count[real]) <= 0)
    # dense entries decode to their original (row, column)
    for k in range(5):
        for bi in range(d["chunk_blk_off"][k], d["chunk_blk_off"][k + 1]):
            e0, e1 = d["blk_e0"][bi], d["blk_e0"][bi + 1]
            assert e1 - e0 >= min_nnz
            pos = d["ent_pos"][e0:e1].astype(np.int64)
            r = d["row_perm"][chunk_ptr[k] + 128 * d["blk_rb"][bi] + (pos >> 8)]
            u = d["colslot_vertex"][64 * d["blk_cb"][bi] + (pos & 255)]
            orig = d["ent_orig"][e0:e1]
            assert np.all((pos & 255) < 64) and np.all((pos >> 8) < 128)
            assert np.array_equal(r, rows_of_entry[orig]) and np.array_equal(u, col[orig])
            seen[orig] += 1
    assert np.all(seen == 1)
    # blocks are sorted by (row chunk, row block, column block)
    for k in range(5):
        s0, s1 = d["chunk_blk_off"][k], d["chunk_blk_off"][k + 1]
        key = d["blk_rb"][s0:s1].astype(np.int64) * (1 << 32) + d["blk_cb"][s0:s1]
        assert np.all(np.diff(key) > 0)
    # an unreachable share leaves the plan inactive
    off = g.gnnstage_dense_plan(row_ptr, col, chunk_ptr, min_nnz, 1.1)
    assert all(len(v) == 0 for k, v in off.items() if k != "min_nnz_used")


def _items_per_chunk(d, K, item_blocks):
    """Items of every chunk: runs of at most item_blocks consecutive blocks of one row block."""
    out = []
    for k in range(K):
        rb = d["blk_rb"][d["chunk_blk_off"][k]:d["chunk_blk_off"][k + 1]]
        out.append(int(sum(-(-c // item_blocks) for c in np.bincount(rb) if c > 0)) if len(rb) else 0)
    return out


def test_dense_plan_threshold_per_chunk_by_rounds_of_workgroups():
    """A chunk whose items at the low threshold fit one round keeps it; a chunk with more items climbs a 5 % ladder
    until it fits, at most to the other threshold; the blocks of every chunk are exactly those of an uncapped plan
    built with that chunk's threshold."""
    g = _lib()
    row_ptr, col = make_graph(CONFIGS["c1_s"])
    n = len(row_ptr) - 1
    K = 5
    chunk_ptr = np.array([0, n // 2, n // 2 + n // 8, n // 2 + n // 4, n // 2 + 3 * n // 8, n], dtype=np.int64)  # one heavy chunk
    low, high = 6, 30
    free = g.gnnstage_dense_plan(row_ptr, col, chunk_ptr, low, 0.0)
    assert list(free["min_nnz_used"]) == [low] * K
    items = _items_per_chunk(free, K, 4)
    limit = sorted(items)[-2]                 # all chunks but the heaviest fit
    assert items[0] == max(items) > limit > 0
    capped = g.gnnstage_dense_plan(row_ptr, col, chunk_ptr, low, 0.0, item_blocks=4, max_items=limit, min_nnz_many=high)
    t0 = int(capped["min_nnz_used"][0])
    assert list(capped["min_nnz_used"][1:]) == [low] * (K - 1) and low < t0 <= high
    ladder = [low]
    while ladder[-1] < t0:
        ladder.append(max(ladder[-1] + 1, int(ladder[-1] * 1.05)))
    assert ladder[-1] == t0 or t0 == high                                     # a rung of the ladder, or its end
    strict = g.gnnstage_dense_plan(row_ptr, col, chunk_ptr, t0, 0.0)
    if t0 < high:                                                             # the first rung that fits
        assert _items_per_chunk(strict, K, 4)[0] <= limit
        assert _items_per_chunk(g.gnnstage_dense_plan(row_ptr, col, chunk_ptr, ladder[-2], 0.0), K, 4)[0] > limit
    never = g.gnnstage_dense_plan(row_ptr, col, chunk_ptr, low, 0.0, item_blocks=4, max_items=1, min_nnz_many=high)
    assert list(never["min_nnz_used"]) == [high] * K                          # nothing fits: the other threshold
    for k in range(K):
        ref = strict if k == 0 else free
        a0, a1 = capped["chunk_blk_off"][k], capped["chunk_blk_off"][k + 1]
        r0, r1 = ref["chunk_blk_off"][k], ref["chunk_blk_off"][k + 1]
        assert a1 - a0 == r1 - r0
        assert np.array_equal(capped["blk_rb"][a0:a1], ref["blk_rb"][r0:r1]) and np.array_equal(capped["blk_cb"][a0:a1], ref["blk_cb"][r0:r1])
        ea, er = capped["blk_e0"], ref["blk_e0"]
        assert np.array_equal(np.diff(ea[a0:a1 + 1]), np.diff(er[r0:r1 + 1]))
        assert np.array_equal(capped["ent_orig"][ea[a0]:ea[a1]], ref["ent_orig"][er[r0]:er[r1]])
        assert np.array_equal(capped["ent_pos"][ea[a0]:ea[a1]], ref["ent_pos"][er[r0]:er[r1]])
    # every entry still exactly once: dense entries + remainder
    seen = np.zeros(row_ptr[-1], dtype=np.int32)
    seen[capped["rem_orig"]] += 1
    seen[capped["ent_orig"]] += 1
    assert np.all(seen == 1)
    same = g.gnnstage_dense_plan(row_ptr, col, chunk_ptr, low, 0.0, item_blocks=4, max_items=max(items), min_nnz_many=high)
    assert list(same["min_nnz_used"]) == [low] * K and np.array_equal(same["blk_e0"], free["blk_e0"])


def test_benchmark_graph_stays_near_the_low_threshold_in_every_chunk():
    """configs[1] with the stage's own settings (3.4 % of a block's cells, items of 32 blocks, 1.1 x 512 workgroups of
    two column halves): every chunk's launch fits one round, two thirds of the entries are dense."""
    g = _lib()
    w = CONFIGS["c1"]
    row_ptr, col = make_graph(w)
    n = len(row_ptr) - 1
    K = w.n_chunks
    chunk_ptr = (np.arange(K + 1, dtype=np.int64) * n) // K
    low, high, max_items = 128 * 64 * 34 // 1000, 128 * 64 // 20, 2 * 256 * 11 // 10 // 2
    d = g.gnnstage_dense_plan(row_ptr, col, chunk_ptr, low, 0.2, item_blocks=32, max_items=max_items, min_nnz_many=high)
    assert all(low <= t <= 1.1 * low for t in d["min_nnz_used"]) and low in d["min_nnz_used"]
    items = _items_per_chunk(d, K, 32)
    assert max(items) <= max_items and min(items) > 0.8 * max_items      # one round, and a full one
    assert 0.6 < d["blk_e0"][-1] / len(col) < 0.75


def _desc(g, **over):
    n = 6
    row_ptr = np.array([0, 1, 2, 3, 4, 5, 6], dtype=np.int64)
    col = np.arange(6, dtype=np.int32)
    chunk_ptr = np.array([0, 3, 6], dtype=np.int64)
    dims = np.array([4, 4], dtype=np.int32)
    d = g.binding.gnnstage_desc()
    d.n_vertices, d.nnz = n, 6
    d.row_ptr, d.col_idx = row_ptr.ctypes.data, col.ctypes.data
    d.n_chunks, d.chunk_ptr = 2, chunk_ptr.ctypes.data
    d.n_layers, d.dims = 1, dims.ctypes.data
    keep = [row_ptr, col, chunk_ptr, dims]
    for k, v in over.items():
        setattr(d, k, v)
    return d, keep


def test_workspace_size_and_validation_without_a_gpu():
    g = _lib()
    d, keep = _desc(g)
    size = g.lib.gnnstage_workspace_size(C.byref(d))
    assert size > 0 and size % 256 == 0
    bad, keep2 = _desc(g, n_chunks=0)
    assert g.lib.gnnstage_workspace_size(C.byref(bad)) == 0
    assert b"n_chunks" in g.lib.gnnstage_last_error(None)
    bad, keep3 = _desc(g, dtype=7)
    assert g.lib.gnnstage_workspace_size(C.byref(bad)) == 0
    # create() rejects a descriptor with missing buffers before any device call
    h = C.c_void_p(None)
    assert g.lib.gnnstage_create(C.byref(d), C.byref(h)) == -1 and h.value is None
    assert g.lib.gnnstage_create(None, C.byref(h)) == -1
    assert g.lib.stage_forward_chunk(None, 0, 0, None) == -1
    assert g.lib.update_history(None, None) == -1
    assert g.lib.gnnstage_destroy(None) == -1


def test_generated_graphs_are_symmetric_sorted_and_reproducible():
    w = CONFIGS["c3_s"]
    a_ptr, a_col = make_graph(w)
    b_ptr, b_col = make_graph(w)
    assert np.array_equal(a_ptr, b_ptr) and np.array_equal(a_col, b_col)
    g = _lib()
    t_ptr, t_row, _ = g.gnnstage_plan_transpose(a_ptr, a_col)
    assert np.array_equal(t_ptr, a_ptr) and np.array_equal(t_row, a_col)  # symmetric
    n = len(a_ptr) - 1
    rows = np.repeat(np.arange(n), np.diff(a_ptr))
    key = rows.astype(np.int64) * n + a_col
    assert np.all(np.diff(key) > 0)  # sorted, no duplicates
    has_loop = np.zeros(n, dtype=bool)
    has_loop[rows[rows == a_col]] = True
    assert has_loop.all()


def test_bench_refuses_more_than_one_gpu():
    """The build covers one pipeline stage on one GPU: asking the benchmark for more ends with a message, before any GPU work."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and "--gpus must be 1" in r.stderr
    assert r.stdout.strip() == ""  # no result line
