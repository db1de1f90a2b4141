"""Seeded draft-tree topologies and token fills.

The paper's decoding trees are static per model family, deeper and wider along
higher-probability branches, with depth up to 8 and up to 20 children at the root
(Appendix "Tree Structure"); the figures that give the exact trees are not
available, so trees here come from a best-first expansion over random path scores
with a per-depth branching list, which has the same character.

Node 0 is the root (the token the target model produced last, whose K/V is not yet
cached); every other node holds one draft token.  Nodes are numbered depth-major
(BFS), so parent[i] < i."""
import heapq
import numpy as np


def gen_prefix(seed: int, length: int, vocab: int) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(key=[seed, 7001]))
    return rng.integers(0, vocab, size=length, dtype=np.int32)


def tree_depths(parent) -> np.ndarray:
    d = np.zeros(len(parent), dtype=np.int32)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return d


def chain_tree(n: int):
    parent = np.arange(-1, n - 1, dtype=np.int32)
    return parent, np.arange(n, dtype=np.int32)


def random_branching(seed: int, n_nodes: int, max_depth: int = 8, lo: int = 1, hi: int = 8):
    """Per-level branching drawn uniformly in [lo, hi]; redrawn until the full tree
    would have at least n_nodes nodes."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 7002]))
    while True:
        br = [int(b) for b in rng.integers(lo, hi + 1, size=max_depth)]
        total, level = 1, 1
        for b in br:
            level *= b
            total += level
        if total >= n_nodes:
            return br


def gen_tree(seed: int, n_nodes: int, branching, plant_len: int = 0):
    """Topology of the n_nodes best nodes (root included) of the tree in which a node
    at depth dep has branching[dep] children.  A child's score is its parent's score
    times U(0,1); the first child along one path down to depth plant_len gets score
    1 so that this path is always kept.  Returns (parent, depth, planted) with
    planted[j] = index of the planted node at depth j (planted[0] = 0)."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 7003]))
    # heap entries: (-score, creation order, parent creation id, depth, planted flag)
    heap = [(-1.0, 0, -1, 0, True)]
    created = 1
    kept = []  # (creation id, parent creation id, depth, planted)
    while heap and len(kept) < n_nodes:
        neg, cid, pcid, dep, planted = heapq.heappop(heap)
        kept.append((cid, pcid, dep, planted))
        if dep < len(branching):
            for c in range(branching[dep]):
                is_pl = planted and c == 0 and dep < plant_len
                sc = -neg * (1.0 if is_pl else float(rng.random()))
                heapq.heappush(heap, (-sc, created, cid, dep + 1, is_pl))
                created += 1
    if len(kept) < n_nodes:
        raise ValueError("branching list yields fewer nodes than requested")
    kept.sort(key=lambda e: (e[2], e[0]))  # depth-major, creation order within a depth
    new_id = {e[0]: i for i, e in enumerate(kept)}
    parent = np.array([-1 if e[1] < 0 else new_id[e[1]] for e in kept], dtype=np.int32)
    depth = np.array([e[2] for e in kept], dtype=np.int32)
    planted = [i for i, e in enumerate(kept) if e[3]]
    planted.sort(key=lambda i: depth[i])
    assert len(planted) == plant_len + 1
    return parent, depth, np.array(planted, dtype=np.int32)


def fill_tokens(seed: int, parent, vocab: int, root_token: int, planted=None, plant_tokens=None,
                avoid=None) -> np.ndarray:
    """Uniform random tokens, siblings distinct.  planted nodes 1.. receive
    plant_tokens; avoid[i] (optional, per node) lists tokens node i must not take."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 7004]))
    n = len(parent)
    tok = np.zeros(n, dtype=np.int32)
    tok[0] = root_token
    fixed = {}
    if planted is not None and plant_tokens is not None:
        for j in range(1, len(planted)):
            fixed[int(planted[j])] = int(plant_tokens[j - 1])
    used = {}  # parent -> set of tokens of its children
    for i, t in fixed.items():
        used.setdefault(int(parent[i]), set()).add(t)
    for i in range(1, n):
        if i in fixed:
            tok[i] = fixed[i]
            continue
        taken = used.setdefault(int(parent[i]), set())
        while True:
            t = int(rng.integers(0, vocab))
            if t in taken or (avoid is not None and t in avoid[i]):
                continue
            break
        taken.add(t)
        tok[i] = t
    return tok


def sibling_ranks(parent) -> np.ndarray:
    """rank[i] = position of node i among the children of its parent, in index order (0 for the
    root).  In a static decoding tree the child of rank r stands for the drafter's r-th most
    likely token at that place (Appendix "Tree Structure")."""
    n = len(parent)
    rank = np.zeros(n, dtype=np.int32)
    seen = {}
    for i in range(1, n):
        p = int(parent[i])
        rank[i] = seen.get(p, 0)
        seen[p] = rank[i] + 1
    return rank
