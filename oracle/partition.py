"""Per-partition index structures (oracle side; test infrastructure).

Section III: each worker q owns a subset of the nodes, computes every layer for them, and needs the
activations of remote neighbours ("boundary" nodes of their owners). This module turns a global CSR
shift operator and a node->partition map into, for every partition:

    local_gid      ascending global ids of the nodes it owns                         [n_local]
    halo_gid       distinct remote nodes referenced by its rows, ordered by
                   (owner partition, global id)                                      [n_halo]
    halo_owner_ptr halo slots of owner p are halo_owner_ptr[p]:halo_owner_ptr[p+1]   [P+1]
    rowptr/colidx/vals   its row block; column c < n_local is local row c, column
                   n_local + s is halo slot s; columns ascending within a row
    t_rowptr/t_colidx/t_vals  the transpose: row c (local or halo) lists the local rows i with
                   S[i, c] != 0, ascending in i
    boundary_rows  ascending local rows that at least one other partition references [n_boundary]
    halo_src_row   position of each halo node in its owner's boundary_rows           [n_halo]
    halo_zrow      the same, offset by the boundary counts of the partitions before
                   the owner (row in the concatenated compressed buffer)             [n_halo]

    halo_row_offset number of halo rows of the partitions before this one: first row of this
                   partition in the concatenation of all partitions' halo rows

The exchange unit is the distinct (node, destination partition) pair, not the edge.

returned_row_map gives the owners' view of the backward exchange (Section III: in the backward pass the
errors of remote nodes travel from the consumers back to the owners).
"""
from __future__ import annotations

import dataclasses

import numpy as np


@dataclasses.dataclass
class Partition:
    q: int
    n_local: int
    n_halo: int
    local_gid: np.ndarray
    halo_gid: np.ndarray
    halo_owner_ptr: np.ndarray
    rowptr: np.ndarray
    colidx: np.ndarray
    vals: np.ndarray
    t_rowptr: np.ndarray
    t_colidx: np.ndarray
    t_vals: np.ndarray
    boundary_rows: np.ndarray = None
    halo_src_row: np.ndarray = None
    halo_zrow: np.ndarray = None
    z_row_offset: int = 0
    halo_row_offset: int = -1        # filled by build_partitions when all partitions are built

    @property
    def n_boundary(self) -> int:
        return int(self.boundary_rows.shape[0])

    @property
    def nnz(self) -> int:
        return int(self.colidx.shape[0])


def build_partitions(n: int, rowptr: np.ndarray, colidx: np.ndarray, vals: np.ndarray,
                     part: np.ndarray, n_parts: int, only=None) -> list[Partition]:
    """All partitions' structures, or just those listed in `only` (same values, less work)."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    colidx = np.asarray(colidx, dtype=np.int64)
    part = np.asarray(part, dtype=np.int64)
    local_index = np.empty(n, dtype=np.int64)          # position of each node inside its owner
    locals_of = []
    for q in range(n_parts):
        mine = np.nonzero(part == q)[0]
        local_index[mine] = np.arange(mine.shape[0])
        locals_of.append(mine)

    # boundary nodes: referenced by a row that another partition owns
    row_owner = np.repeat(part, np.diff(rowptr))
    needed_by_others = np.zeros(n, dtype=bool)
    needed_by_others[colidx[row_owner != part[colidx]]] = True
    del row_owner
    boundary_index = np.full(n, -1, dtype=np.int64)    # position inside the owner's boundary list
    boundary_rows, offsets = [], []
    offset = 0
    for p in range(n_parts):
        mine = locals_of[p]
        brow = np.nonzero(needed_by_others[mine])[0]
        boundary_rows.append(brow.astype(np.int32))
        boundary_index[mine[brow]] = np.arange(brow.shape[0])
        offsets.append(offset)
        offset += brow.shape[0]
    offsets = np.asarray(offsets, dtype=np.int64)

    parts: list[Partition] = []
    for q in (range(n_parts) if only is None else only):
        mine = locals_of[q]
        n_local = mine.shape[0]
        lens = rowptr[mine + 1] - rowptr[mine]
        my_rowptr = np.concatenate(([0], np.cumsum(lens))).astype(np.int64)
        nnz = int(my_rowptr[-1])
        # gather this row block's global entries
        entry = np.repeat(rowptr[mine] - my_rowptr[:-1], lens) + np.arange(nnz, dtype=np.int64)
        gcol = colidx[entry]
        val = np.asarray(vals)[entry]
        row_of = np.repeat(np.arange(n_local, dtype=np.int64), lens)
        remote = part[gcol] != q

        halo = np.unique(gcol[remote])
        order = np.lexsort((halo, part[halo]))          # by owner, then by id
        halo = halo[order]
        n_halo = halo.shape[0]
        owner_ptr = np.searchsorted(part[halo], np.arange(n_parts + 1), side="left").astype(np.int64)

        slot = np.empty(n, dtype=np.int64)              # scratch map gid -> halo slot (valid on halo only)
        slot[halo] = np.arange(n_halo)
        newcol = np.where(remote, n_local + slot[gcol], local_index[gcol])
        # ascending columns inside each row
        perm = np.lexsort((newcol, row_of))
        newcol, val, row_of_sorted = newcol[perm], val[perm], row_of[perm]
        assert np.array_equal(row_of_sorted, row_of)

        # transpose: sort entries by (column, row)
        tperm = np.lexsort((row_of, newcol))
        t_counts = np.bincount(newcol, minlength=n_local + n_halo)
        t_rowptr = np.concatenate(([0], np.cumsum(t_counts))).astype(np.int64)

        src = boundary_index[halo]
        assert (src >= 0).all()
        parts.append(Partition(
            q=q, n_local=int(n_local), n_halo=int(n_halo),
            local_gid=mine.astype(np.int32), halo_gid=halo.astype(np.int32),
            halo_owner_ptr=owner_ptr.astype(np.int32),
            rowptr=my_rowptr.astype(np.int32), colidx=newcol.astype(np.int32), vals=val.astype(np.float32),
            t_rowptr=t_rowptr.astype(np.int32), t_colidx=row_of[tperm].astype(np.int32),
            t_vals=val[tperm].astype(np.float32),
            boundary_rows=boundary_rows[q], halo_src_row=src.astype(np.int32),
            halo_zrow=(src + offsets[part[halo]]).astype(np.int32), z_row_offset=int(offsets[q])))
    if only is None:
        before = 0
        for p in parts:
            p.halo_row_offset = before
            before += p.n_halo
    return parts


def returned_row_map(parts: list[Partition]):
    """Owner side of the backward exchange. All consumers' returned rows form one array: consumer q's halo slot
    s is row halo_row_offset[q] + s. For every owner p returns (ret_ptr, ret_src): ret_src[ret_ptr[b]:ret_ptr[b+1]]
    are the rows of that array that carry the errors of p's boundary row b, one per consumer that has the node in
    its halo, consumers in ascending order. `parts` must be all partitions, in order."""
    n_parts = len(parts)
    assert [p.q for p in parts] == list(range(n_parts))
    # one record per exchanged (node, consumer) pair: owner, owner's boundary row, consumer, row of the array
    owner = np.concatenate([np.repeat(np.arange(n_parts), np.diff(p.halo_owner_ptr)) for p in parts])
    brow = np.concatenate([p.halo_src_row.astype(np.int64) for p in parts])
    consumer = np.concatenate([np.full(p.n_halo, p.q, dtype=np.int64) for p in parts])
    row = np.arange(owner.shape[0], dtype=np.int64)        # consumers are concatenated in order: offset + slot
    order = np.lexsort((consumer, brow, owner))            # by owner, then boundary row, then consumer
    owner, brow, row = owner[order], brow[order], row[order]
    first = np.searchsorted(owner, np.arange(n_parts + 1))
    out = []
    for p in parts:
        mine = slice(int(first[p.q]), int(first[p.q + 1]))
        ptr = np.searchsorted(brow[mine], np.arange(p.n_boundary + 1))
        out.append((ptr.astype(np.int32), row[mine].astype(np.int32)))
    return out


def exchanged_rows(parts: list[Partition]) -> int:
    """Number of (node, destination partition) pairs = rows handed off per layer and direction."""
    return int(sum(p.n_halo for p in parts))
