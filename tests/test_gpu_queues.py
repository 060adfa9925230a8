"""GPU check of the attention kernel's work queues (white box).

`prism_sparse_attn` builds, in the caller's workspace behind the V^T image, one queue entry per
(q-head, q-block) row and a plan of eight queue segments.  The parity tests see a broken queue
only through the rows they sample, so this test reads the tables back after a call and checks
what must hold for every row: each row is listed exactly once, with the clamped bounds of its
list and its first valid entry; the segments tile the table; every queue was pulled to its end;
inside a queue the (phase, length class) groups come in order; the queues hold about equal work.

The offsets below restate the workspace layout of prism_attn.hip (V^T image, then the int4
entries, two int32 tables of h*N, class counts, part counts, the 32-int plan, and for whole
blocks of 128 tokens an fp16 copy of the image with one range flag per kv block; every piece
aligned to 256 bytes).  They are not part of the C ABI: this file changes with that layout.
"""
import numpy as np
import pytest
import torch

from paper_2602_08426_amd import binding as pb

pytestmark = pytest.mark.gpu

N_CLASSES = 11


def _align(x, a=256):
    return (x + a - 1) // a * a


def _layout(h, hkv, N, B, L=None):
    rows = h * N
    off = {}
    o = 0
    off["image"] = o
    o = _align(o + hkv * N * B * 128 * 2)
    off["items"] = o
    o = _align(o + rows * 16)
    off["row_rank"] = o
    o = _align(o + rows * 4)
    off["row_part"] = o
    o = _align(o + rows * 4)
    off["bins"] = o
    o = _align(o + 2 * h * N_CLASSES * 4)
    off["parts"] = o
    o = _align(o + hkv * N_CLASSES * 8 * 4)
    off["plan"] = o
    o = _align(o + 32 * 4)
    if B == 128 and (L is None or L % 128 == 0):
        # whole blocks of 128 tokens: a second V^T image in fp16 and one range flag per kv block
        off["image16"] = o
        o = _align(o + hkv * N * B * 128 * 2)
        off["range_flags"] = o
        o = _align(o + hkv * N * 4)
    if B == 64 and N % 2 == 0:
        # an even number of 64-token blocks: a second plan over pairs of q-blocks (pair kernel)
        off["pair_items"] = o
        o = _align(o + rows // 2 * 16)
        off["pair_plan"] = o
        o = _align(o + 32 * 4)
    off["total"] = o
    return off


def _length_class(n):
    if n <= 1:
        return N_CLASSES - 1
    k = int(n - 1).bit_length() - 1                 # n in (2^k, 2^(k+1)]
    return 0 if k > 9 else 9 - k


@pytest.mark.parametrize("h,hkv,L,B,bidir,seed", [
    (8, 2, 128 * 96, 128, False, 0),     # 768 rows: eight queues, one phase
    (4, 4, 64 * 300 + 17, 64, False, 1),  # ragged last block, group size 1
    (6, 2, 128 * 50, 128, True, 2),      # bidirectional lists
    (1, 1, 128 * 3, 128, False, 3),      # fewer rows than XCDs: a single queue
    (16, 8, 128 * 1024, 128, False, 4),  # 128K tokens: four phases of two kv heads
])
def test_every_row_is_queued_once_and_the_queues_are_balanced(h, hkv, L, B, bidir, seed):
    print(f"case h={h}/{hkv} L={L} B={B} bidirectional={bidir}", flush=True)
    rng = np.random.default_rng(seed)
    N = (L + B - 1) // B
    flags = pb.PRISM_FLAG_BIDIRECTIONAL if bidir else 0
    params = pb.make_params(h, hkv, L, B, flags=flags)
    lay = _layout(h, hkv, N, B, L)
    assert pb.prism_sparse_attn_workspace_bytes(params) == lay["total"]

    # heads of very different density, some empty rows, some entries that the kernel must skip
    lists = []
    for hq in range(h):
        density = [0.02, 0.1, 0.3, 0.9][hq % 4]
        for u in range(N):
            vmax = N - 1 if bidir else u
            n = rng.binomial(vmax + 1, density)
            if rng.random() < 0.03:
                n = 0
            cols = np.sort(rng.choice(vmax + 1, size=n, replace=False)).astype(np.int32)
            if n and rng.random() < 0.05:
                cols[0] = -1                                  # garbage in front: skipped
            lists.append(cols)
    lens = np.array([len(c) for c in lists])
    row_ptr = np.zeros(h * N + 1, np.int32)
    row_ptr[1:] = np.cumsum(lens)
    col_idx = np.concatenate(lists + [np.zeros(1, np.int32)]).astype(np.int32)
    nnz = int(row_ptr[-1])

    q = torch.zeros((h, L, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((hkv, L, 128), dtype=torch.bfloat16, device="cuda")
    v = torch.zeros((hkv, L, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(q)
    ws = pb.alloc_workspace(lay["total"])
    rp_d, ci_d = torch.from_numpy(row_ptr).cuda(), torch.from_numpy(col_idx).cuda()
    pb.prism_sparse_attn(params, q, k, v, rp_d, ci_d, nnz, out, None, ws)
    torch.cuda.synchronize()
    raw = ws.cpu().numpy()

    rows = h * N
    items = raw[lay["items"]:lay["items"] + rows * 16].view(np.int32).reshape(rows, 4)
    plan = raw[lay["plan"]:lay["plan"] + 96].view(np.int32)
    start, length, pulled = plan[0:8], plan[8:16], plan[16:24]

    # the segments tile the table, and every queue was pulled past its end
    assert length.sum() == rows
    np.testing.assert_array_equal(start, np.cumsum(length) - length)
    assert (pulled >= length).all()
    n_queues = 8 if min(rows, 512 if B == 128 else 1024) >= 8 else 1
    assert (length[n_queues:] == 0).all()

    # every row exactly once, with its own list bounds and first valid entry
    hq, u = items[:, 0], items[:, 1] & 0xFFFF
    v0, it0, end = (items[:, 1] >> 16) & 0xFFFF, items[:, 2], items[:, 3]
    assert ((hq >= 0) & (hq < h) & (u < N)).all()
    r = hq * N + u
    assert len(np.unique(r)) == rows
    np.testing.assert_array_equal(end, row_ptr[r + 1])
    for e in rng.choice(rows, size=min(rows, 4000), replace=False):
        cols = lists[r[e]]
        vmax = N - 1 if bidir else u[e]
        valid = np.nonzero((cols >= 0) & (cols <= vmax))[0]
        if len(valid):
            assert it0[e] == row_ptr[r[e]] + valid[0] and v0[e] == cols[valid[0]], (e, r[e])
        else:
            assert it0[e] == end[e], (e, r[e])

    # order inside a queue: (phase, class) never goes back; inside a group q-heads ascend and,
    # inside a head, q-blocks descend
    head_bytes = L * 128 * 2 * 2
    hpp = max(1, (160 << 20) // head_bytes)
    g = h // hkv
    work = []
    for x in range(8):
        seg = slice(start[x], start[x] + length[x])
        ph = (hq[seg] // g) // hpp
        cls = np.array([_length_class(n) for n in lens[r[seg]]])
        key = ph * N_CLASSES + cls
        assert (np.diff(key) >= 0).all(), f"queue {x}: groups out of order"
        same = np.diff(key) == 0
        dh = np.diff(hq[seg])
        assert (dh[same] >= 0).all(), f"queue {x}: q-heads out of order"
        du = np.diff(u[seg].astype(np.int64))
        assert (du[same & (dh == 0)] < 0).all(), f"queue {x}: q-blocks out of order"
        work.append(int((lens[r[seg]] + 1).sum()))
    work = np.array(work[:n_queues])
    print(f"  work per queue {work.tolist()}", flush=True)
    if n_queues == 8 and rows >= 512:
        # a part boundary can be off by one row per (phase, class) group
        slack = (lens.max() + 1) * N_CLASSES * max(1, -(-hkv // hpp))
        assert work.max() - work.min() <= slack, (work, slack)


@pytest.mark.parametrize("h,hkv,N,dirty", [(4, 2, 40, False), (8, 2, 300, False), (4, 2, 40, True)])
def test_pair_plan_at_block_64(h, hkv, N, dirty):
    """B = 64 with an even number of blocks: the pair kernel's plan holds every pair of q-blocks once,
    its queues are pulled past their ends when the lists are clean, and not at all when a list holds an
    entry to skip (then the plain kernel takes the call and its plan is the one that is used up)."""
    rng = np.random.default_rng(5 + N)
    B, L = 64, 64 * N
    params = pb.make_params(h, hkv, L, B, flags=pb.PRISM_FLAG_PAIR_KERNEL)
    lay = _layout(h, hkv, N, B, L)
    assert pb.prism_sparse_attn_workspace_bytes(params) == lay["total"]
    lists = []
    for hq in range(h):
        for u in range(N):
            n = rng.binomial(u + 1, [0.05, 0.3, 0.8, 0.15][hq % 4])
            lists.append(np.sort(rng.choice(u + 1, size=n, replace=False)).astype(np.int32))
    if dirty:
        lists[h * N // 2] = np.array([N + 3], np.int32)
    lens = np.array([len(c) for c in lists])
    row_ptr = np.zeros(h * N + 1, np.int32)
    row_ptr[1:] = np.cumsum(lens)
    col_idx = np.concatenate(lists + [np.zeros(1, np.int32)]).astype(np.int32)
    q = torch.zeros((h, L, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((hkv, L, 128), dtype=torch.bfloat16, device="cuda")
    v = torch.zeros((hkv, L, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(q)
    ws = pb.alloc_workspace(lay["total"])
    pb.prism_sparse_attn(params, q, k, v, torch.from_numpy(row_ptr).cuda(), torch.from_numpy(col_idx).cuda(),
                         int(row_ptr[-1]), out, None, ws)
    torch.cuda.synchronize()
    raw = ws.cpu().numpy()
    rows = h * N // 2
    items = raw[lay["pair_items"]:lay["pair_items"] + rows * 16].view(np.int32).reshape(rows, 4)
    pplan = raw[lay["pair_plan"]:lay["pair_plan"] + 96].view(np.int32)
    plan = raw[lay["plan"]:lay["plan"] + 128].view(np.int32)
    start, length, pulled = pplan[0:8], pplan[8:16], pplan[16:24]
    assert length.sum() == rows
    np.testing.assert_array_equal(start, np.cumsum(length) - length)
    hq, up = items[:, 0], items[:, 1] & 0xFFFF
    assert len(np.unique(hq * (N // 2) + up)) == rows
    r0 = hq * N + 2 * up
    np.testing.assert_array_equal(items[:, 2], row_ptr[r0])
    np.testing.assert_array_equal(items[:, 3], row_ptr[r0 + 2])
    assert plan[24] == (1 if dirty else 0)
    if dirty:
        assert (pulled == 0).all() and (plan[16:24] >= plan[8:16]).all()
    else:
        assert (pulled >= length).all() and (plan[16:24] == 0).all()
