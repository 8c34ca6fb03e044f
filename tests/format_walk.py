"""Test helpers: read a built HB-CSF representation back through the C ABI and walk it on the CPU.

Two independent walks, both in fp64 numpy / Python:
  * walk_algorithms: Algorithms "CSF-MTTKRP", "CSL-MTTKRP" and "COO-MTTKRP" applied to the three
    groups as stored (segments -> tmp -> times the middle row -> slice row).  Validates the
    builder against the oracle (Eq. 7 = Eq. 8).
  * emulate_kernels: the GPU kernels' own schedule (runs of L nonzeros per lane group, end marks,
    plain stores for slices inside one run, atomic merges otherwise, partial rows carried across
    units) with every output row tracked, so a row that is stored twice, stored and also merged,
    or never defined is reported.
"""
import numpy as np

from paper_1904_03329_amd import binding as B


def read_mode(h, mode, order):
    st = B.get_stats(h, mode)
    fmt = {"stats": st, "order": order, "L": st["fiber_threshold"], "level_mode": st["level_mode"][:order]}
    for gname, g in (("coo", 0), ("csl", 1), ("csf", 2)):
        d = {"ind": {}, "ptr": {}, "run": {}}
        for lvl in range(order):
            for key, aid in (("ind", B.ARR_IND), ("ptr", B.ARR_PTR), ("run", B.ARR_RUNFIRST)):
                try:
                    d[key][lvl] = B.host_array(h, mode, g, lvl, aid)
                except B.HbcsfError:
                    pass
        d["val"] = B.host_array(h, mode, g, 0, B.ARR_VAL)
        d["nnz"] = st["group_nnz"][g]
        d["slices"] = st["group_slices"][g]
        fmt[gname] = d
    fmt["owned"] = B.host_array(h, mode, 0, 0, B.ARR_OWNED_BITS)
    coo = fmt["coo"]
    fmt["coo_row_flags"] = coo["nnz"] > 0 and len(coo["ind"][0]) == 0
    if fmt["coo_row_flags"]:
        # no stored root indices: the nonzeros are in row order and the row bitmap says which rows they are
        bits = B.host_array(h, mode, 0, 0, B.ARR_COO_BITS)
        rows = np.flatnonzero(np.unpackbits(bits.view(np.uint8), bitorder="little"))
        assert rows.shape[0] == coo["nnz"]
        coo["ind"][0] = rows.astype(np.uint32)
    return fmt


def expand_to_coo(fmt):
    """All nonzeros of the three groups as (tree-level index arrays, values)."""
    order = fmt["order"]
    cols = [[] for _ in range(order)]
    vals = []
    coo = fmt["coo"]
    if coo["nnz"]:
        for l in range(order):
            cols[l].append(coo["ind"][l][: coo["nnz"]])
        vals.append(coo["val"][: coo["nnz"]])
    csl = fmt["csl"]
    if csl["nnz"]:
        n = csl["slices"]
        ptr = csl["ptr"][0][: n + 1].astype(np.int64)
        cols[0].append(np.repeat(csl["ind"][0][:n] & 0x7FFFFFFF, np.diff(ptr)))
        for l in range(1, order):
            cols[l].append(csl["ind"][l][: csl["nnz"]])
        vals.append(csl["val"][: csl["nnz"]])
    csf = fmt["csf"]
    if csf["nnz"]:
        for l in range(order - 1):
            n = len(csf["ind"][l]) - 1
            ptr = csf["ptr"][l][: n + 1].astype(np.int64)
            cols[l].append(np.repeat(csf["ind"][l][:n] & 0x7FFFFFFF, np.diff(ptr)))
        cols[order - 1].append(csf["ind"][order - 1][: csf["nnz"]])
        vals.append(csf["val"][: csf["nnz"]])
    if not vals:
        return [np.zeros(0, np.uint32) for _ in range(order)], np.zeros(0, np.float32)
    return [np.concatenate(c) for c in cols], np.concatenate(vals)


def walk_algorithms(fmt, factors, rows, rank):
    """fp64 result of running the three per-group algorithms over the stored arrays."""
    order = fmt["order"]
    fac = [None] + [factors[fmt["level_mode"][l]].astype(np.float64) for l in range(1, order)]
    y = np.zeros((rows, rank))
    coo = fmt["coo"]
    for z in range(coo["nnz"]):
        p = np.full(rank, float(coo["val"][z]))
        for l in range(1, order):
            p = p * fac[l][coo["ind"][l][z]]
        y[coo["ind"][0][z]] += p
    csl = fmt["csl"]
    for s in range(csl["slices"]):
        i = csl["ind"][0][s] & 0x7FFFFFFF
        for z in range(csl["ptr"][0][s], csl["ptr"][0][s + 1]):
            p = np.full(rank, float(csl["val"][z]))
            for l in range(1, order):
                p = p * fac[l][csl["ind"][l][z]]
            y[i] += p
    csf = fmt["csf"]
    if csf["nnz"]:
        leaf = order - 1
        # deepest fiber level: tmp = sum v * leafRow, then times this level's row
        n = len(csf["ind"][leaf - 1]) - 1
        part = np.zeros((n, rank))
        for f in range(n):
            tmp = np.zeros(rank)
            for z in range(csf["ptr"][leaf - 1][f], csf["ptr"][leaf - 1][f + 1]):
                tmp += float(csf["val"][z]) * fac[leaf][csf["ind"][leaf][z]]
            part[f] = tmp * fac[leaf - 1][csf["ind"][leaf - 1][f]]
        starts = csf["ptr"][leaf - 1][:n].astype(np.int64)
        for l in range(leaf - 2, -1, -1):
            n_up = len(csf["ind"][l]) - 1
            up = np.zeros((n_up, rank))
            owner = np.searchsorted(csf["ptr"][l][: n_up + 1].astype(np.int64), starts, side="right") - 1
            np.add.at(up, owner, part)
            if l > 0:
                up *= fac[l][csf["ind"][l][:n_up]]
                part, starts = up, csf["ptr"][l][:n_up].astype(np.int64)
            else:
                np.add.at(y, (csf["ind"][0][:n_up] & 0x7FFFFFFF).astype(np.int64), up)
    return y


class _Rows:
    """Output rows with bookkeeping of how each was defined."""

    def __init__(self, rows, rank, owned_bits):
        self.y = np.zeros((rows, rank))
        self.owned = np.array([(owned_bits[r >> 5] >> (r & 31)) & 1 for r in range(rows)], dtype=bool)
        self.stored = np.zeros(rows, dtype=np.int64)
        self.merged = np.zeros(rows, dtype=np.int64)

    def store(self, row, acc):
        assert self.owned[row], f"plain store to row {row} that the define kernel zeroes"
        self.stored[row] += 1
        self.y[row] = acc

    def atomic(self, row, acc):
        assert not self.owned[row], f"atomic merge into row {row} that is never zeroed"
        self.merged[row] += 1
        self.y[row] += acc

    def check(self):
        assert np.all(self.stored[self.owned] == 1), "an owned row was not stored exactly once"
        assert np.all(self.stored[~self.owned] == 0)


def _marks(n_rec, ptr, ind, z0, lo, hi, owned_aware):
    out = np.zeros(n_rec, dtype=np.int64)
    for s in range(lo, hi):
        p = int(ptr[s + 1]) - 1 - z0
        assert 0 <= p < n_rec, "an end mark falls outside its unit"
        v = int(ind[s])
        out[p] = ((v & 0x7FFFFFFF) + 1) | (v & 0x80000000) if owned_aware else v + 1
    return out


def _emulate_group(kind, g, fmt, fac, rows_obj, rank, lane_groups, units_per_wave):
    order, L = fmt["order"], fmt["L"]
    nnz = g["nnz"]
    if nnz == 0:
        return
    runs = (nnz + L - 1) // L
    n_units = (runs + lane_groups - 1) // lane_groups
    run0 = g["run"][0]
    ind0 = g["ind"][0]
    leaf = order - 1
    n_waves = (n_units + units_per_wave - 1) // units_per_wave
    for w in range(n_waves):
        acc = [np.zeros(rank) for _ in range(lane_groups)]
        pend = [False] * lane_groups
        pend_row = [0] * lane_groups
        for u in range(w * units_per_wave, min((w + 1) * units_per_wave, n_units)):
            r0 = u * lane_groups
            z0 = r0 * L
            rn = min(r0 + lane_groups, runs)
            n_rec = lane_groups * L
            slice_mark = _marks(n_rec, g["ptr"][0], ind0, z0, int(run0[r0]), int(run0[rn]), True)
            seg_mark = {}
            if kind == "csf":
                for l in range(1, order - 1):
                    seg_mark[l] = _marks(n_rec, g["ptr"][l], g["ind"][l], z0, int(g["run"][l][r0]),
                                         int(g["run"][l][rn]), False)
            for q in range(lane_groups):
                r = r0 + q
                if r >= runs:
                    continue
                ng = min(L, nnz - r * L)
                head = int(ind0[run0[r]]) & 0x7FFFFFFF
                tail = int(ind0[run0[r + 1]]) & 0x7FFFFFFF
                if pend[q] and pend_row[q] != head:
                    rows_obj.atomic(pend_row[q], acc[q])
                    acc[q] = np.zeros(rank)
                tmp = {l: np.zeros(rank) for l in range(1, order)}
                is_open = True
                for t in range(ng):
                    p = q * L + t
                    z = z0 + p
                    v = float(g["val"][z])
                    if kind == "csl":
                        pr = np.full(rank, v)
                        for l in range(1, order):
                            pr = pr * fac[l][g["ind"][l][z]]
                        acc[q] = acc[q] + pr
                    else:
                        tmp[leaf] = tmp[leaf] + v * fac[leaf][g["ind"][leaf][z]]
                        for l in range(leaf - 1, 0, -1):  # deepest fiber level first
                            m = int(seg_mark[l][p])
                            if not m:
                                break
                            contrib = tmp[l + 1] * fac[l][m - 1]
                            tmp[l + 1] = np.zeros(rank)
                            if l == 1:
                                acc[q] = acc[q] + contrib
                            else:
                                tmp[l] = tmp[l] + contrib
                    m = int(slice_mark[p])
                    if m:
                        row = (m & 0x7FFFFFFF) - 1
                        if m & 0x80000000:
                            rows_obj.store(row, acc[q])
                        else:
                            rows_obj.atomic(row, acc[q])
                        acc[q] = np.zeros(rank)
                    is_open = m == 0
                pend[q] = is_open
                pend_row[q] = tail
        for q in range(lane_groups):
            if pend[q]:
                rows_obj.atomic(pend_row[q], acc[q])


def emulate_kernels(fmt, factors, rows, rank, units_per_wave=2):
    order = fmt["order"]
    lane_groups = 64 // (rank // 4)
    fac = [None] + [factors[fmt["level_mode"][l]].astype(np.float64) for l in range(1, order)]
    out = _Rows(rows, rank, fmt["owned"])
    coo = fmt["coo"]
    for z in range(coo["nnz"]):
        p = np.full(rank, float(coo["val"][z]))
        for l in range(1, order):
            p = p * fac[l][coo["ind"][l][z]]
        out.store(int(coo["ind"][0][z]), p)
    _emulate_group("csl", fmt["csl"], fmt, fac, out, rank, lane_groups, units_per_wave)
    _emulate_group("csf", fmt["csf"], fmt, fac, out, rank, lane_groups, units_per_wave)
    out.check()
    return out.y


def emulate_nonroot(fmt, factors, target_mode, rows, rank):
    """The schedule of the single-representation kernel (target mode at a tree level T >= 1 of another mode's
    B-CSF representation), in fp64: every lane group walks its run of L nonzeros with START marks (index + 1 at the
    first nonzero of each slice / fiber segment), keeps the rows of the levels above the leaf, and adds
        out(i_T) += (product of the rows above level T) * sum over the level-T segment of v * (rows below level T)
    at the end of each level-T segment (T = leaf: per nonzero).  Only the CSF group may hold nonzeros."""
    order, L = fmt["order"], fmt["L"]
    assert fmt["coo"]["nnz"] == 0 and fmt["csl"]["nnz"] == 0
    g = fmt["csf"]
    T = fmt["level_mode"].index(target_mode)
    assert T >= 1
    leaf = order - 1
    fac = [factors[fmt["level_mode"][l]].astype(np.float64) for l in range(order)]
    out = np.zeros((rows, rank))
    nnz = g["nnz"]
    runs = (nnz + L - 1) // L
    starts = {}
    for l in range(order - 1):
        n = len(g["ind"][l]) - 1
        mark = np.zeros(nnz, dtype=np.int64)
        mark[g["ptr"][l][:n].astype(np.int64)] = (g["ind"][l][:n].astype(np.int64) & 0x7FFFFFFF) + 1
        starts[l] = mark
    for r in range(runs):
        z0, z1 = r * L, min((r + 1) * L, nnz)
        head = int(g["ind"][0][g["run"][0][r]]) & 0x7FFFFFFF
        cur = [None] * order
        cur[0] = head
        acc, is_open = np.zeros(rank), False
        up = dn = None
        for z in range(z0, z1):
            marks = [int(starts[l][z]) for l in range(order - 1)]
            if any(marks):
                if T < leaf and marks[T] and is_open:
                    out[cur[T]] += acc * up
                    acc = np.zeros(rank)
                for l in range(order - 1):
                    if marks[l]:
                        cur[l] = marks[l] - 1
                        if l == T:
                            is_open = True
                assert all(cur[l] is not None for l in range(order - 1)), "a level has no index yet: missing start mark"
                up = np.ones(rank)
                for l in range(T):
                    up = up * fac[l][cur[l]]
                dn = np.ones(rank)
                for l in range(T + 1, leaf):
                    dn = dn * fac[l][cur[l]]
            v = float(g["val"][z])
            k = int(g["ind"][leaf][z])
            if T == leaf:
                out[k] += v * up
            else:
                acc = acc + v * fac[leaf][k] * dn
        if T < leaf and is_open:
            out[cur[T]] += acc * up
    return out
