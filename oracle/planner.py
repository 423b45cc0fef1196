"""Oracle task planner -- TEST INFRASTRUCTURE ONLY (never imported by the product path).

Cleave's PS performs task generation per GEMM node: it cuts A into row blocks
and B into column blocks; a task is one (row block, column block) pair and
yields the matching sub-block of the output (Sec. 3.2 "Seamless training";
Sec. 4.1 "Search space of GEMM").  The shard assignment has to cover the
output exactly, with no redundant work (Sec. 4.1, coverage constraint
sum_k alpha_k*beta_k = m*q) and no empty shard (Sec. 4.1, zero-task
constraint).

On top of the paper's row/column cut, the inner dimension is cut into S
contiguous chunks (the K-split); the S partial blocks of one output tile are
summed afterwards by the aggregator.  S = 1 is the paper's own case.

Everything below is integer bookkeeping written as plain loops.

Rules (the readings where the paper is silent):
  * uniform tiling: ceil(M/tile_m) x ceil(N/tile_n) tiles, last row/column of
    tiles clipped, never padded (padding would break the coverage constraint);
  * explicit tiling: horizontal bands of given heights that sum to M; each band
    is cut into columns of given widths that sum to N; every tile carries its
    own split count S;
  * K-split: kc = ceil(K/S); chunk s is [s*kc, min((s+1)*kc, K)); a split that
    would leave an empty chunk ((S-1)*kc >= K) is rejected;
  * order: tile rows (bands) outermost, tile columns next, split index s
    innermost; tile_id is the running tile index, a task's index is its
    position in that order;
  * partial_off is the running sum of m_len*n_len over the preceding tasks, so
    every task owns a contiguous row-major m_len x n_len block and the S
    blocks of one tile are adjacent.
"""
import numpy as np

# Byte layout of one task record: mirrors `cleave_task` in include/cleave.h
# (an interface both sides have to agree on; 64 bytes, little endian).
TASK_DTYPE = np.dtype([
    ("gemm_id", "<u4"), ("tile_id", "<u4"),
    ("m0", "<u4"), ("m_len", "<u4"),
    ("n0", "<u4"), ("n_len", "<u4"),
    ("k0", "<u4"), ("k_len", "<u4"),
    ("ksplit_idx", "<u4"), ("ksplit_cnt", "<u4"),
    ("partial_off", "<u8"),
    ("flags", "<u4"), ("reserved0", "<u4"), ("reserved1", "<u4"), ("reserved2", "<u4"),
])
assert TASK_DTYPE.itemsize == 64


class PlanError(ValueError):
    pass


def _ceil_div(a, b):
    return -(-a // b)


def k_chunks(K, S):
    """[(k0, k_len)] for the S contiguous chunks of the inner dimension."""
    if K < 1 or S < 1:
        raise PlanError("K and S must be positive")
    kc = _ceil_div(K, S)
    if (S - 1) * kc >= K:
        raise PlanError("K-split %d of K=%d leaves an empty chunk" % (S, K))
    out = []
    for s in range(S):
        k0 = s * kc
        out.append((k0, min(kc, K - k0)))
    return out


def _emit(tiles, K, gemm_id):
    """tiles: list of (m0, m_len, n0, n_len, S) in canonical order."""
    records = []
    off = 0
    for tile_id, (m0, m_len, n0, n_len, S) in enumerate(tiles):
        if m_len < 1 or n_len < 1:
            raise PlanError("empty tile")
        for s, (k0, k_len) in enumerate(k_chunks(K, S)):
            records.append((gemm_id, tile_id, m0, m_len, n0, n_len, k0, k_len,
                            s, S, off, 0, 0, 0, 0))
            off += m_len * n_len
    tasks = np.array(records, dtype=TASK_DTYPE)
    return tasks, off


def plan_uniform(M, N, K, tile_m, tile_n, ksplit, gemm_id=0):
    """Returns (tasks, partial_elems) for the uniform tiling."""
    if min(M, N, K, tile_m, tile_n, ksplit) < 1:
        raise PlanError("all sizes must be positive")
    tiles = []
    for r in range(_ceil_div(M, tile_m)):
        m0 = r * tile_m
        m_len = min(tile_m, M - m0)
        for c in range(_ceil_div(N, tile_n)):
            n0 = c * tile_n
            n_len = min(tile_n, N - n0)
            tiles.append((m0, m_len, n0, n_len, ksplit))
    return _emit(tiles, K, gemm_id)


def plan_explicit(M, N, K, band_h, col_w, ksplit_per_tile, gemm_id=0):
    """band_h: heights of the row bands (sum M).  col_w: one list of column
    widths per band (each sums to N).  ksplit_per_tile: S per tile, band-major.
    Returns (tasks, partial_elems)."""
    if min(M, N, K) < 1:
        raise PlanError("all sizes must be positive")
    if len(band_h) < 1 or len(col_w) != len(band_h):
        raise PlanError("need one column list per band")
    if sum(band_h) != M:
        raise PlanError("band heights do not sum to M")
    tiles = []
    m0 = 0
    t = 0
    for h, widths in zip(band_h, col_w):
        if h < 1 or len(widths) < 1:
            raise PlanError("empty band")
        if sum(widths) != N:
            raise PlanError("column widths do not sum to N")
        n0 = 0
        for w in widths:
            if w < 1:
                raise PlanError("empty column")
            if t >= len(ksplit_per_tile):
                raise PlanError("too few K-split entries")
            tiles.append((m0, h, n0, w, int(ksplit_per_tile[t])))
            n0 += w
            t += 1
        m0 += h
    if t != len(ksplit_per_tile):
        raise PlanError("too many K-split entries")
    return _emit(tiles, K, gemm_id)


def plan_batched(M, N, K, tile_m, tile_n, ksplit, n_batch):
    """A batch of n_batch independent GEMMs of one shape in one task list (the
    per-head score GEMMs of Sec. 3.1, Table "GEMM shapes": Q x K^T is
    1024 x 128 x 1024, one per sequence and head).  GEMM g contributes the
    uniform plan of a single GEMM with gemm_id = g; its tile ids start at 0
    again; partial offsets continue through the whole list.
    Returns (tasks, partial_elems)."""
    if n_batch < 1:
        raise PlanError("empty batch")
    one, elems = plan_uniform(M, N, K, tile_m, tile_n, ksplit, 0)
    parts = []
    for g in range(n_batch):
        t = one.copy()
        t["gemm_id"] = g
        t["partial_off"] += g * elems
        parts.append(t)
    return np.concatenate(parts), elems * n_batch


# ---------------------------------------------------------------------------
# Invariant checkers (the constraints the paper fixes for any valid plan).
# ---------------------------------------------------------------------------

def check_plan_invariants(tasks, M, N, K):
    """Raises AssertionError unless the plan satisfies the paper's constraints:
    no empty task; per output tile the K chunks partition [0, K); the tiles are
    pairwise disjoint and their areas sum to M*N (exact cover without redundant
    work); total flops equal 2*M*N*K; partial blocks are packed back to back."""
    assert len(tasks) > 0
    vol = 0
    area_by_tile = {}
    kcover = {}
    off = 0
    for t in tasks:
        m0, ml, n0, nl, k0, kl = (int(t[f]) for f in ("m0", "m_len", "n0", "n_len", "k0", "k_len"))
        assert ml >= 1 and nl >= 1 and kl >= 1
        assert m0 + ml <= M and n0 + nl <= N and k0 + kl <= K
        assert int(t["partial_off"]) == off
        off += ml * nl
        vol += ml * nl * kl
        tid = int(t["tile_id"])
        rect = (m0, ml, n0, nl)
        assert area_by_tile.setdefault(tid, rect) == rect
        kcover.setdefault(tid, []).append((int(t["ksplit_idx"]), int(t["ksplit_cnt"]), k0, kl))
    assert vol == M * N * K
    assert sum(r[1] * r[3] for r in area_by_tile.values()) == M * N
    for tid, chunks in kcover.items():
        S = chunks[0][1]
        assert [c[0] for c in chunks] == list(range(S))
        assert all(c[1] == S for c in chunks)
        pos = 0
        for _, _, k0, kl in chunks:
            assert k0 == pos
            pos += kl
        assert pos == K
    # Pairwise disjoint rectangles: sweep over sorted rows is overkill here;
    # with equal total area, disjointness <=> every cell covered at most once.
    rects = sorted(area_by_tile.values())
    for a in range(len(rects)):
        am0, aml, an0, anl = rects[a]
        for b in range(a + 1, len(rects)):
            bm0, bml, bn0, bnl = rects[b]
            if bm0 >= am0 + aml:
                break
            rows_overlap = bm0 < am0 + aml and am0 < bm0 + bml
            cols_overlap = bn0 < an0 + anl and an0 < bn0 + bnl
            assert not (rows_overlap and cols_overlap)
    return True
