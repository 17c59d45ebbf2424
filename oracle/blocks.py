"""Oracle (test infrastructure): Binary Block Matrix, run index, sparse block list, packed mask bits.

Definitions (paper Sec. 4 "Binary Block Masking", "Dense Binary Block Masking"; Appendix A, the block-sum
formulation) with the readings this build fixes where the paper is silent:

* the mask is zero-padded to nbr*Br x nbc*Bc with nbr = ceil(N/Br), nbc = ceil(N/Bc) (the paper assumes
  divisibility); a block that contains padding can therefore never be "filled with ones"; the mask may be
  rectangular, [Mb, Nq, Nk] (nbr from Nq, nbc from Nk), for queries that attend a longer key/value cache;
* cnt[i][j]  = number of non-zero elements of block (i, j);   BinBlkMat[i][j] = (cnt > 0);
* class[i][j] = 0 if cnt == 0, 2 if cnt == Br*Bc, else 1;
* total_ones[i], offset[i] = length and first block of the LONGEST run of consecutive class-2 blocks in
  block row i (leftmost on ties; (0, 0) if none) -- "blocks filled with ones" is read as all-ones blocks,
  which is what lets the attention step skip the element mask inside the run;
* nz_lo / nz_hi / nz_cnt = first non-zero block, one past the last, and their number ((0,0,0) if none);
* sparse list: row_ptr[i+1]-row_ptr[i] = nz_cnt[i]; col_idx ascending, bit 31 set iff the block is class 2;
  plane m of col_idx starts at m*nbr*nbc (fixed capacity), row_ptr is per plane and starts at 0;
* column list (for the backward pass, which walks the queries of a key block): col_ptr[j+1]-col_ptr[j] = number of
  non-zero blocks of block column j; row_idx ascending block rows, bit 31 set iff the block is class 2; plane m of
  row_idx starts at m*nbr*nbc, col_ptr is per plane and starts at 0;
* packed[m][w][r] bit t (little-endian in a uint64) = (mask[m][r][64*w + t] != 0), zero beyond column N.
"""
import numpy as np


def block_counts(mask, Br, Bc):
    """mask [Mb,Nq,Nk] -> int64 [Mb,nbr,nbc] non-zero counts per block of the zero-padded mask."""
    Mb, N, Nk = mask.shape
    nbr, nbc = -(-N // Br), -(-Nk // Bc)
    out = np.zeros((Mb, nbr, nbc), dtype=np.int64)
    for m in range(Mb):
        pad = np.zeros((nbr * Br, nbc * Bc), dtype=np.uint8)
        pad[:N, :Nk] = mask[m] != 0
        out[m] = pad.reshape(nbr, Br, nbc, Bc).sum(axis=(1, 3), dtype=np.int64)
    return out


def block_class(mask, Br, Bc):
    cnt = block_counts(mask, Br, Bc)
    cls = np.ones(cnt.shape, dtype=np.uint8)
    cls[cnt == 0] = 0
    cls[cnt == Br * Bc] = 2
    return cls


def bin_blk_mat(mask, Br, Bc):
    """The paper's BinBlkMat via its 'any element non-zero' wording (not via the counts)."""
    Mb, N, Nk = mask.shape
    nbr, nbc = -(-N // Br), -(-Nk // Bc)
    out = np.zeros((Mb, nbr, nbc), dtype=np.uint8)
    for m in range(Mb):
        for i in range(nbr):
            for j in range(nbc):
                out[m, i, j] = 1 if np.any(mask[m, i * Br:(i + 1) * Br, j * Bc:(j + 1) * Bc]) else 0
    return out


def run_index(cls):
    """cls uint8 [Mb,nbr,nbc] -> dict of int32 [Mb,nbr] arrays: offset, total_ones, nz_lo, nz_hi, nz_cnt."""
    Mb, nbr, nbc = cls.shape
    res = {k: np.zeros((Mb, nbr), dtype=np.int32) for k in ("offset", "total_ones", "nz_lo", "nz_hi", "nz_cnt")}
    for m in range(Mb):
        for i in range(nbr):
            row = cls[m, i]
            best_len, best_start, j = 0, 0, 0
            while j < nbc:
                if row[j] == 2:
                    s = j
                    while j < nbc and row[j] == 2:
                        j += 1
                    if j - s > best_len:
                        best_len, best_start = j - s, s
                else:
                    j += 1
            res["offset"][m, i], res["total_ones"][m, i] = best_start, best_len
            nz = [j for j in range(nbc) if row[j] != 0]
            if nz:
                res["nz_lo"][m, i], res["nz_hi"][m, i], res["nz_cnt"][m, i] = nz[0], nz[-1] + 1, len(nz)
    return res


def sparse_index(cls):
    """cls [Mb,nbr,nbc] -> row_ptr int32 [Mb,nbr+1], col_idx uint32 [Mb*nbr*nbc] (unused tail entries = 0)."""
    Mb, nbr, nbc = cls.shape
    row_ptr = np.zeros((Mb, nbr + 1), dtype=np.int32)
    col_idx = np.zeros(Mb * nbr * nbc, dtype=np.uint32)
    for m in range(Mb):
        p = 0
        for i in range(nbr):
            for j in range(nbc):
                c = cls[m, i, j]
                if c != 0:
                    col_idx[m * nbr * nbc + p] = j | (0x80000000 if c == 2 else 0)
                    p += 1
            row_ptr[m, i + 1] = p
    return row_ptr, col_idx


def column_index(cls):
    """cls [Mb,nbr,nbc] -> col_ptr int32 [Mb,nbc+1], row_idx uint32 [Mb*nbr*nbc] (unused tail entries = 0)."""
    Mb, nbr, nbc = cls.shape
    col_ptr = np.zeros((Mb, nbc + 1), dtype=np.int32)
    row_idx = np.zeros(Mb * nbr * nbc, dtype=np.uint32)
    for m in range(Mb):
        p = 0
        for j in range(nbc):
            for i in range(nbr):
                c = cls[m, i, j]
                if c != 0:
                    row_idx[m * nbr * nbc + p] = i | (0x80000000 if c == 2 else 0)
                    p += 1
            col_ptr[m, j + 1] = p
    return col_ptr, row_idx


def packed_bits(mask):
    """mask [Mb,N,Nk] -> uint64 [Mb, ceil(Nk/64), N]: word-column major, bit t of word (w, r) = mask[r][64w+t] != 0."""
    Mb, N, Nk = mask.shape
    W = -(-Nk // 64)
    out = np.zeros((Mb, W, N), dtype=np.uint64)
    for m in range(Mb):
        nzr, nzc = np.nonzero(mask[m])
        np.bitwise_or.at(out[m], (nzc // 64, nzr), np.uint64(1) << (nzc % 64).astype(np.uint64))
    return out


SCHED_PART_BASE = 8
SCHED_PART_INTS = 8
SCHED_MIN_SPLIT = 32
SCHED_MAX_SORT_ROWS = 4096
SCHED_ROW_INTS = 4
SCHED_GROUP_ROWS = 4


def schedule(row_ptr, col_idx):
    """Split schedule of the list mode (this build's own layout, stated in the library header).

    row_ptr int32 [Mb, nbr+1], col_idx uint32 [Mb*nbr*nbc] (as sparse_index returns them) -> int32 array of 8 + 12*Mb*nbr entries: [0] parts,
    [1] split threshold T = max(32, 2*ceil(mean list length of the non-empty rows)), [2] cut rows, [3..7] 0, then
    8 ints per part in (row, part) order: row (= plane*nbr + block row), first entry (position in the plane's list),
    entries, part, parts of the row, number of the row's first part, index of the row among the cut rows, the list
    entry at the part's first position (as int32).
    A row with n > T entries is cut into ceil(n/T) parts of ceil(n/parts) entries (the last part takes the rest);
    rows with n <= T are not listed.  Table entries past the last part are unspecified.  The last 4*Mb*nbr entries
    are one record of 4 ints per (plane, rank), in the order in which the block rows of a plane are started: the rows
    are taken in groups of 4 consecutive rows if T = 32, i.e. while rows are short (neighbours share most of their
    key/value tiles, so they should run at the same time), else one by one (with long rows the plain longest-first
    order balances the tail better); the groups are ordered by the list length of their longest row, longest first
    (ties: the group of higher rows first), the rows inside a group by list length, longest first (ties: higher row
    first).  Planes of more than 4096
    block rows are listed from the last row to the first instead.  A record holds the block row, the position of its
    first list entry in the plane's list, its number of entries, and its first list entry (-1 if it has none)."""
    Mb, nbr1 = row_ptr.shape
    nbr = nbr1 - 1
    counts = [int(row_ptr[m, i + 1] - row_ptr[m, i]) for m in range(Mb) for i in range(nbr)]
    nonempty = sum(1 for c in counts if c > 0)
    mean = -(-sum(counts) // nonempty) if nonempty else 0
    T = max(SCHED_MIN_SPLIT, 2 * mean)
    order_base = SCHED_PART_BASE + SCHED_PART_INTS * Mb * nbr
    out = np.zeros(order_base + SCHED_ROW_INTS * Mb * nbr, dtype=np.int32)
    lists = np.asarray(col_idx, dtype=np.uint32).reshape(Mb, -1)
    entry = lambda m, pos: int(lists[m, pos].astype(np.int32))
    for m in range(Mb):
        rows = list(range(nbr - 1, -1, -1))
        if nbr <= SCHED_MAX_SORT_ROWS:
            length = lambda i: counts[m * nbr + i]
            gsz = SCHED_GROUP_ROWS if T == SCHED_MIN_SPLIT else 1
            groups = [list(range(a, min(a + gsz, nbr))) for a in range(0, nbr, gsz)]
            groups.sort(key=lambda g: (-max(length(i) for i in g), -g[0]))      # group of the longest row first; ties: higher rows
            rows = [i for g in groups for i in sorted(g, key=lambda i: (-length(i), -i))]
        for rank, i in enumerate(rows):
            o = order_base + SCHED_ROW_INTS * (m * nbr + rank)
            c = counts[m * nbr + i]
            out[o:o + 4] = (i, int(row_ptr[m, i]), c, entry(m, int(row_ptr[m, i])) if c > 0 else -1)
    q, rho = 0, 0
    for r, c in enumerate(counts):
        if c <= T:
            continue
        parts = -(-c // T)
        chunk = -(-c // parts)
        for k in range(parts):
            first = int(row_ptr[r // nbr, r % nbr]) + k * chunk
            o = SCHED_PART_BASE + SCHED_PART_INTS * (q + k)
            out[o:o + 8] = (r, first, min(chunk, c - k * chunk), k, parts, q, rho, entry(r // nbr, first))
        q += parts
        rho += 1
    out[0], out[1], out[2] = q, T, rho
    return out


COL_SCHED_MIN_SPLIT = 16


def column_schedule(col_ptr, row_idx):
    """Split schedule and launch order of the backward pass's column walk (this build's own layout, stated in the
    library header).

    col_ptr int32 [Mb, nbc+1], row_idx uint32 [Mb*nbr*nbc] (as column_index returns them) -> int32 array of
    8 + 12*Mb*nbc entries: [0] parts, [1] split threshold T = max(16, 2*ceil(mean list length of the non-empty
    columns)), [2] cut columns, [3..7] 0, then 8 ints per part in (column, part) order: column (= plane*nbc + block
    column), first entry (position in the plane's list), entries, part, parts of the column, number of the column's
    first part, index of the column among the cut columns, the list entry at the part's first position (as int32).
    A column with n > T entries is cut into ceil(n/T) parts of ceil(n/parts) entries (the last part takes the rest);
    columns with n <= T are not listed.  Table entries past the last part are unspecified.  The last 4*Mb*nbc entries
    are one record of 4 ints per (plane, rank) in the order in which the block columns of a plane are started: by list
    length, longest first (ties: the higher column first); planes of more than 4096 block columns are listed from the
    last column to the first instead.  A record holds the block column, the position of its first list entry in the
    plane's list, its number of entries, and its first list entry (-1 if it has none)."""
    Mb, nbc1 = col_ptr.shape
    nbc = nbc1 - 1
    counts = [int(col_ptr[m, j + 1] - col_ptr[m, j]) for m in range(Mb) for j in range(nbc)]
    nonempty = sum(1 for c in counts if c > 0)
    mean = -(-sum(counts) // nonempty) if nonempty else 0
    T = max(COL_SCHED_MIN_SPLIT, 2 * mean)
    order_base = SCHED_PART_BASE + SCHED_PART_INTS * Mb * nbc
    out = np.zeros(order_base + SCHED_ROW_INTS * Mb * nbc, dtype=np.int32)
    lists = np.asarray(row_idx, dtype=np.uint32).reshape(Mb, -1)
    entry = lambda m, pos: int(lists[m, pos].astype(np.int32))
    for m in range(Mb):
        cols = list(range(nbc - 1, -1, -1))
        if nbc <= SCHED_MAX_SORT_ROWS:
            cols.sort(key=lambda j: -counts[m * nbc + j])           # stable: equal lengths keep the higher column first
        for rank, j in enumerate(cols):
            o = order_base + SCHED_ROW_INTS * (m * nbc + rank)
            c = counts[m * nbc + j]
            out[o:o + 4] = (j, int(col_ptr[m, j]), c, entry(m, int(col_ptr[m, j])) if c > 0 else -1)
    q, rho = 0, 0
    for col, c in enumerate(counts):
        if c <= T:
            continue
        parts = -(-c // T)
        chunk = -(-c // parts)
        m = col // nbc
        for k in range(parts):
            first = int(col_ptr[m, col % nbc]) + k * chunk
            o = SCHED_PART_BASE + SCHED_PART_INTS * (q + k)
            out[o:o + 8] = (col, first, min(chunk, c - k * chunk), k, parts, q, rho, entry(m, first))
        q += parts
        rho += 1
    out[0], out[1], out[2] = q, T, rho
    return out


def block_index(mask, Br, Bc):
    """Everything the preprocessing stage produces, as a dict."""
    cls = block_class(mask, Br, Bc)
    idx = dict(cls=cls, bin_blk_mat=(cls != 0).astype(np.uint8))
    idx.update(run_index(cls))
    idx["row_ptr"], idx["col_idx"] = sparse_index(cls)
    idx["sched"] = schedule(idx["row_ptr"], idx["col_idx"])
    idx["col_ptr"], idx["row_idx"] = column_index(cls)
    idx["col_sched"] = column_schedule(idx["col_ptr"], idx["row_idx"])
    return idx
