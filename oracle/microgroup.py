"""Oracle: micro-group plan - batch one rank's same-shape matrices.

Test infrastructure only (see the package docstring).

The paper's micro-groups (Sec. 4, Algorithm 2) fuse the tensors of one
All-to-All; the per-rank step built here batches the matrices a rank owns so
that one launch handles several of them, which needs equal shapes.  The rule,
stated once here and in the design notes:

1. take the ids with owner == rank in ascending id;
2. a shape class is the exact triple (rows, cols, dtype) - a matrix and its
   transpose are different classes;
3. classes are ordered by per-matrix numel descending, ties by the smallest
   member id (the deterministic (W(p), ID_p) ordering of Algorithm 2, Phase 1,
   read as a stable sort);
4. each class, members in ascending id, is cut into consecutive chunks of at
   most ``max_mats`` matrices (0 = no cap) and at most ``cmax_bytes`` bytes of
   bf16 matrix data (0 = no cap); a single matrix above ``cmax_bytes`` is an
   error, as in Algorithm 3 ("single item exceeds C_max").
"""
from __future__ import annotations


def microgroup_plan(rows, cols, dtype, owner, rank, max_mats=8, cmax_bytes=0):
    """Returns a list of groups, each a list of matrix ids."""
    if max_mats < 0 or cmax_bytes < 0:
        raise ValueError("caps must be non-negative")
    owned = [p for p in range(len(rows)) if owner[p] == rank]
    classes = {}
    for p in owned:
        classes.setdefault((int(rows[p]), int(cols[p]), int(dtype[p])), []).append(p)
    keys = sorted(classes, key=lambda k: (-(k[0] * k[1]), classes[k][0]))
    groups = []
    for key in keys:
        one_bytes = 2 * key[0] * key[1]
        if cmax_bytes and one_bytes > cmax_bytes:
            raise ValueError("single matrix exceeds cmax_bytes")
        cur = []
        for p in classes[key]:
            full = (max_mats and len(cur) == max_mats) or \
                   (cmax_bytes and (len(cur) + 1) * one_bytes > cmax_bytes)
            if cur and full:
                groups.append(cur)
                cur = []
            cur.append(p)
        if cur:
            groups.append(cur)
    return groups
