"""Plain Python reference of the paper's context index (Section 4 and Section 5, Appendix
algorithms "Context Index Construction via Hierarchical Clustering", "Context Index Tree
Search", "Context Alignment for Prefix Sharing", "Search-Path-Based Request Grouping and
Scheduling").

TEST INFRASTRUCTURE ONLY: imported by the tests and by the CPU-baseline leg of the benchmark.
The C++ library never imports this module and this module imports nothing from it.  Everything
here is written for reading, not for speed: lists, sets, explicit loops, cubic-time clustering.

Where the paper leaves a choice open, the reading taken is stated where it is used.
"""
from __future__ import annotations

from collections import deque
from typing import Dict, List, Optional, Sequence, Tuple


def distance(ci: Sequence[int], cj: Sequence[int], alpha: float) -> float:
    """Context distance (Eq. 1).  Positions are 0-based ranks in the lists; ids within a list
    are distinct.  No shared id: the positional term is taken as 0 (distance 1); two empty
    contexts are at distance 0."""
    if len(ci) == 0 and len(cj) == 0:
        return 0.0
    pos_j = {b: p for p, b in enumerate(cj)}
    shared = [(p, pos_j[b]) for p, b in enumerate(ci) if b in pos_j]
    d = 1.0 - len(shared) / max(len(ci), len(cj))
    if shared:
        d += alpha * sum(abs(p - q) for p, q in shared) / len(shared)
    return d


def distance_matrix(contexts: Sequence[Sequence[int]], alpha: float) -> List[List[float]]:
    n = len(contexts)
    return [[0.0 if i == j else distance(contexts[i], contexts[j], alpha) for j in range(n)] for i in range(n)]


def linkage(D: Sequence[Sequence[float]]) -> List[Tuple[int, int, float, int]]:
    """Agglomerative clustering of n points from their distance matrix (construction
    algorithm, phase 1, "Z <- Linkage(D)").

    Reading: the paper names no linkage rule; average linkage (the distance between two
    clusters is the mean of the point distances between them) is taken.  Each step merges the
    two active clusters at the smallest distance; among equal distances the pair with the
    smallest lower id wins, then the smallest higher id.  Points have ids 0..n-1, the cluster
    made by step t has id n + t.  Returns one tuple (id_a, id_b, distance, size) per step with
    id_a < id_b.
    """
    n = len(D)
    dist: Dict[Tuple[int, int], float] = {}
    for i in range(n):
        for j in range(i + 1, n):
            dist[(i, j)] = float(D[i][j])
    size = {i: 1 for i in range(n)}
    active = list(range(n))
    merges = []
    for step in range(n - 1):
        best = None
        for x in range(len(active)):
            for y in range(x + 1, len(active)):
                a, b = active[x], active[y]      # a < b because ids only grow
                key = (dist[(a, b)], a, b)
                if best is None or key < best:
                    best = key
        d, a, b = best
        new = n + step
        for c in active:
            if c != a and c != b:
                dac = dist[(min(a, c), max(a, c))]
                dbc = dist[(min(b, c), max(b, c))]
                dist[(c, new)] = (size[a] * dac + size[b] * dbc) / (size[a] + size[b])
        size[new] = size[a] + size[b]
        active = [c for c in active if c != a and c != b] + [new]
        merges.append((a, b, d, size[new]))
    return merges


class Node:
    """A node of the index: the context (block ids, aligned to the prefix of its parent), its
    children, an access frequency and the clustering distance at which it was created."""

    def __init__(self, docs: Sequence[int], leaf: bool, created_at: float = 0.0):
        self.docs: List[int] = list(docs)
        self.children: List["Node"] = []
        self.parent: Optional["Node"] = None
        self.leaf = leaf
        self.freq = 1 if leaf else 0
        self.created_at = created_at

    def leaves(self) -> int:
        return 1 if self.leaf else sum(c.leaves() for c in self.children)

    def path(self) -> List[int]:
        """Child indices from the root to this node."""
        out = []
        v = self
        while v.parent is not None:
            out.append(v.parent.children.index(v))
            v = v.parent
        return out[::-1]


def _align_to(prefix: Sequence[int], docs: Sequence[int]) -> List[int]:
    """prefix followed by the rest of docs in their own order."""
    p = set(prefix)
    return list(prefix) + [b for b in docs if b not in p]


class ContextIndex:
    """The tree.  `root` has the empty context."""

    def __init__(self, alpha: float):
        self.alpha = alpha
        self.root = Node([], leaf=False)
        self.leaf_of: List[Node] = []     # input context i -> its leaf

    # ---- construction -------------------------------------------------------------------
    @classmethod
    def build(cls, contexts: Sequence[Sequence[int]], alpha: float,
              D: Optional[Sequence[Sequence[float]]] = None) -> "ContextIndex":
        """Index over a batch of contexts.

        Readings: identical contexts (same ids in the same order) share one leaf whose
        frequency counts them, and the clustering runs over the distinct contexts in order of
        first appearance (a duplicate is at distance 0 of its twin, so clustering it
        separately would only recreate the twin).  D, when given, is the distance matrix of the
        distinct contexts; otherwise it is computed with Eq. 1.  A virtual node's context is
        the intersection of its two children's contexts in ascending id order.  Children are
        listed with the larger subtree (more leaves) first, equal sizes in id order.  Virtual
        nodes with an empty context are removed and their children take their place under the
        grandparent; the top of the tree hangs under a root with the empty context.
        """
        idx = cls(alpha)
        uniq: List[Tuple[int, ...]] = []
        where: Dict[Tuple[int, ...], int] = {}
        member = []
        for c in contexts:
            t = tuple(int(b) for b in c)
            if t not in where:
                where[t] = len(uniq)
                uniq.append(t)
            member.append(where[t])
        n = len(uniq)
        if D is None:
            D = distance_matrix(uniq, alpha)
        assert len(D) == n
        nodes: List[Node] = [Node(u, leaf=True) for u in uniq]
        for leaf in nodes:
            leaf.freq = 0
        for m in member:
            nodes[m].freq += 1
        content = [set(u) for u in uniq]          # raw content per cluster id
        for a, b, d, _ in linkage(D):
            inter = content[a] & content[b]
            v = Node(sorted(inter), leaf=False, created_at=d)
            kids = sorted([a, b], key=lambda c: (-nodes[c].leaves(), c))
            for c in kids:
                v.children.append(nodes[c])
                nodes[c].parent = v
            nodes.append(v)
            content.append(inter)
        top = nodes[-1] if n > 0 else None
        if top is not None:
            idx.root.children.append(top)
            top.parent = idx.root
        idx._remove_empty(idx.root)
        # top-down prefix alignment, breadth first
        queue = deque(idx.root.children)
        while queue:
            v = queue.popleft()
            if v.parent is not idx.root and v.parent.docs:
                v.docs = _align_to(v.parent.docs, v.docs)
            queue.extend(v.children)
        idx.leaf_of = [nodes[m] for m in member]
        return idx

    def _remove_empty(self, v: Node) -> None:
        changed = True
        while changed:
            changed = False
            kids: List[Node] = []
            for c in v.children:
                if not c.leaf and not c.docs:
                    kids.extend(c.children)      # grandchildren take the place of c
                    changed = True
                else:
                    kids.append(c)
            v.children = kids
            for c in kids:
                c.parent = v
        for c in v.children:
            if not c.leaf:
                self._remove_empty(c)

    # ---- search ---------------------------------------------------------------------------
    def search(self, C: Sequence[int]) -> Tuple[List[int], Node]:
        """Greedy descent (search algorithm).  At every node the overlapping child at the
        smallest distance from C is taken (first such child among equals).

        Reading of the stopping rule ("stops upon reaching a leaf or when all children are
        equidistant, indicating the longest shared prefix"): the descent stops at the current
        node when even the best child shares no more blocks with C than the current node's own
        context does - going down would not lengthen the shared prefix.  This reproduces the
        paper's worked example (C6 stops at C4); a literal test for equal distances would
        already stop one level higher there, because under Eq. 1 the children {1,2} and {1,4,0}
        of C5 are at the same distance from {2,1,4}.

        The descent also ends at a child that holds blocks C does not have (a partial match):
        nothing below it can be a prefix of C.  Such a node, like a leaf, is returned as the
        match together with the path that leads to it; every node above it on the path has a
        context that C contains completely.
        """
        cset = set(C)
        cur = self.root
        path: List[int] = []
        while cur.children:
            best, best_d = None, None
            for i, ch in enumerate(cur.children):
                if cset.isdisjoint(ch.docs):
                    continue
                d = distance(C, ch.docs, self.alpha)
                if best is None or d < best_d:
                    best, best_d = i, d
            if best is None:
                break
            ch = cur.children[best]
            if len(cset & set(ch.docs)) <= len(cset & set(cur.docs)):
                break
            path.append(best)
            if ch.leaf or not cset.issuperset(ch.docs):
                return path, ch
            cur = ch
        return path, cur

    def insert(self, C: Sequence[int]) -> Tuple[List[int], List[int]]:
        """Searches, aligns (alignment algorithm) and stores a new context.  Returns the
        aligned context and its search path.

        Match = a virtual node whose whole context C contains (or the root): C inherits that
        context as its prefix and becomes the node's last child.  Match = a leaf or a partial
        match: a new virtual node takes its place under the same parent, holding the blocks the
        two share in the order the matched node has them, with the matched node and C as its
        children; the matched node and everything below it stay as they are (they are cached
        in that order).  C is the prefix it inherits followed by its other blocks in their
        original order.  An identical context only raises the leaf's frequency.
        """
        C = [int(b) for b in C]
        cset = set(C)
        path, node = self.search(C)
        if node.leaf and node.docs == _align_to(node.parent.docs, C):
            node.freq += 1
            self.leaf_of.append(node)
            return list(node.docs), path
        if node.leaf or not cset.issuperset(node.docs):
            parent = node.parent
            v = Node([b for b in node.docs if b in cset], leaf=False,
                     created_at=distance(C, node.docs, self.alpha))
            at = parent.children.index(node)
            parent.children[at] = v
            v.parent = parent
            v.children.append(node)
            node.parent = v
            node = v
        aligned = _align_to(node.docs, C)
        for ch in node.children:
            if ch.leaf and ch.docs == aligned:
                ch.freq += 1
                self.leaf_of.append(ch)
                return list(ch.docs), ch.path()
        leaf = Node(aligned, leaf=True)
        leaf.parent = node
        node.children.append(leaf)
        self.leaf_of.append(leaf)
        return list(leaf.docs), leaf.path()

    # ---- views ----------------------------------------------------------------------------
    def aligned(self, i: int) -> List[int]:
        return list(self.leaf_of[i].docs)

    def path(self, i: int) -> List[int]:
        return self.leaf_of[i].path()

    def nodes_bfs(self) -> List[Node]:
        out, queue = [], deque([self.root])
        while queue:
            v = queue.popleft()
            out.append(v)
            queue.extend(v.children)
        return out


def schedule(paths: Sequence[Sequence[int]]) -> List[int]:
    """Execution order from search paths (scheduling algorithm): group by the first path
    element, inside a group longer paths first, larger groups first.  Both sorts are stable, so
    equal keys keep their input order; groups keep the order in which they first appear."""
    groups: Dict[int, List[int]] = {}
    for i, p in enumerate(paths):
        key = p[0] if len(p) else -1
        groups.setdefault(key, []).append(i)
    ordered = []
    for key in groups:                       # insertion order = first appearance
        g = sorted(groups[key], key=lambda i: -len(paths[i]))
        ordered.append(g)
    ordered.sort(key=lambda g: -len(g))
    return [i for g in ordered for i in g]


def prefix_hits(aligned: Sequence[Sequence[int]], order: Sequence[int]) -> List[int]:
    """Blocks of each context that an exact prefix cache holding every earlier context (in
    execution order, nothing evicted) would serve: the longest common prefix with any earlier
    context.  Returned per context, in input order."""
    seen: List[Sequence[int]] = []
    hits = [0] * len(aligned)
    for i in order:
        best = 0
        for s in seen:
            k = 0
            while k < len(s) and k < len(aligned[i]) and s[k] == aligned[i][k]:
                k += 1
            best = max(best, k)
        hits[i] = best
        seen.append(aligned[i])
    return hits
