"""A second, deliberately naive statement of the paper's Algorithm 1 in pure
Python (dict pool, set visited, min/max by scanning), used only to cross-check
the C++ oracle's control flow on tiny inputs.  It consumes precomputed keys, so
it holds none of the distance arithmetic."""


def naive_search(keys, adjacency, entries, ef, pad=0xFFFFFFFF, labels=None, alpha_s=float("inf"), m_s=None,
                 expansions_per_step=1):
    """keys[v] = traversal key of node v.  Returns (sorted pool [(key, id)], n_exp, n_dist)."""
    pool = {}            # id -> expanded?
    visited = set()
    n_exp = n_dist = 0
    degree = len(adjacency[0])
    if m_s is None or m_s <= 0:
        m_s = degree

    def order(v):
        return (float(keys[v]), int(v))

    def insert(v):
        nonlocal n_dist
        n_dist += 1
        pool[v] = False
        if len(pool) > ef:
            worst = max(pool, key=order)
            del pool[worst]

    for e in entries:
        e = int(e)
        if e == pad or e in visited:
            continue
        visited.add(e)
        insert(e)
    while True:
        todo = sorted((v for v, done in pool.items() if not done), key=order)[:expansions_per_step]
        if not todo:
            break
        batch = []
        for u in todo:
            pool[u] = True
            n_exp += 1
            taken = 0
            for slot in range(degree):
                v = int(adjacency[u][slot])
                if v == pad or v in visited:
                    continue
                if labels is not None and not (labels[u][slot] <= alpha_s):
                    continue
                if not (taken < m_s):
                    continue
                visited.add(v)
                batch.append(v)
                taken += 1
        for v in batch:
            insert(v)
    return sorted(order(v) for v in pool), n_exp, n_dist
