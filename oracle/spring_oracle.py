"""Plain-Python oracle of the paper's streaming partitioner (Algorithm 1 and the
edge pass described after it in the section on graph partitioning).

TEST INFRASTRUCTURE ONLY: nothing outside tests/ imports this file.  It exists to
check the compiled partitioner in ``sdt_gen`` that produces partitions with
replicas as a workload; it shares no code with it.  Pure-Python loops over
dictionaries and lists: use it on small graphs.

The algorithm has three steps and an edge pass:

1. node clustering over the edge stream (Alg. 1, node clustering): an endpoint
   seen for the first time opens a cluster whose volume is its degree; when the
   endpoints sit in different clusters whose volumes are both at most tau_vol,
   the endpoint of the cluster with the smaller volume (the first endpoint on
   equality) moves into the other cluster; every node also remembers its
   richest neighbour, the neighbour of largest degree seen so far;
2. cluster merging (Alg. 1, cluster merging): a cluster's representative is the
   member whose richest neighbour has the largest degree; clusters are visited
   from the smallest upwards and a cluster is merged into the cluster of its
   representative's richest neighbour when that is another cluster and the two
   together hold at most beta * |V| / p nodes; a cluster that has grown takes
   its place in the order according to its new size;
3. greedy sorted list scheduling (Alg. 1, assigning clusters to partitions):
   clusters from the largest downwards, each to the partition that holds the
   fewest nodes so far;
4. edge pass: an edge inside a partition belongs to it, an edge across two
   partitions is stored in both, so that a partition holds the full neighbour
   list of every node it owns plus replicas of the outside neighbours.

Where the paper leaves a choice open this file takes these readings:
* ties (equal degrees of richest neighbours, equal cluster sizes, equal
  partition loads) go to the candidate met first: the strict "<" of the
  algorithm keeps the earlier richest neighbour and the earlier representative
  (nodes are scanned in ascending id), clusters of equal size are ordered by
  cluster number, partitions of equal load by index;
* a node that never occurs in the stream (degree 0) forms a cluster of its own
  after the stream, numbered after all streamed clusters in ascending node id;
  it has no richest neighbour and is never a merge source;
* a cluster that absorbed another one is visited (again) at the rank of its new
  size, which always lies ahead of the current position;
* the merge test is the algorithm's "<=" (the prose says "smaller than").
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple


def stream_clustering(n: int, degree: Sequence[int], edges: Sequence[Tuple[int, int]], tau_vol: int):
    """Alg. 1, node clustering.  Returns (cluster[n], volume list, richest[n]); clusters are numbered from 0
    in order of creation, richest[v] = -1 if v has no neighbour.

    Written from the definitions rather than as the algorithm's bookkeeping: a cluster IS its set of
    members, its volume is recomputed as the sum of its members' degrees whenever a decision needs it
    (so no running volume can drift from the membership), and a node's richest neighbour is read off
    the list of neighbours the stream has shown it, once, at the end."""
    members: List[set] = []                  # cluster number -> nodes in it now
    home = [-1] * n                          # node -> its cluster number (-1: not seen yet)
    shown: List[List[int]] = [[] for _ in range(n)]   # node -> neighbours in the order the stream showed them

    def volume(c: int) -> int:
        return sum(degree[x] for x in members[c])

    def join_stream(x: int) -> None:
        if home[x] < 0:
            home[x] = len(members)
            members.append({x})

    for u, v in edges:
        join_stream(u)
        join_stream(v)
        cu, cv = home[u], home[v]
        if cu != cv:
            vol_u, vol_v = volume(cu), volume(cv)
            if vol_u <= tau_vol and vol_v <= tau_vol:
                # the endpoint of the lighter cluster changes sides (the first endpoint when they weigh the same)
                mover, src, dst = (u, cu, cv) if vol_u <= vol_v else (v, cv, cu)
                members[src].discard(mover)
                members[dst].add(mover)
                home[mover] = dst
        shown[u].append(v)
        shown[v].append(u)
    for x in range(n):                       # nodes the stream never showed
        join_stream(x)
    richest = [-1] * n
    for x in range(n):
        if shown[x]:
            top = max(degree[w] for w in shown[x])
            richest[x] = next(w for w in shown[x] if degree[w] == top)     # the first one shown among equals
    return home, [volume(c) for c in range(len(members))], richest


def merge_clusters(n: int, degree: Sequence[int], cluster: Sequence[int], richest: Sequence[int], p: int,
                   beta: float) -> List[int]:
    """Alg. 1, cluster merging.  Returns the merged cluster number of every node
    (a surviving cluster keeps its number)."""
    members: Dict[int, List[int]] = {}
    for v in range(n):
        members.setdefault(cluster[v], []).append(v)

    def rich_degree(v: int) -> int:          # degree of v's richest neighbour; -1 if it has none
        return degree[richest[v]] if richest[v] >= 0 else -1

    rep: Dict[int, int] = {}
    for v in range(n):                       # representative: first node with the top richest neighbour
        c = cluster[v]
        if richest[v] >= 0 and (c not in rep or rich_degree(rep[c]) < rich_degree(v)):
            rep[c] = v

    where = list(cluster)                    # current cluster of every node
    limit = beta * n / p
    pending = set(members)
    while pending:
        i = min(pending, key=lambda c: (len(members[c]), c))
        pending.discard(i)
        if i not in rep:
            continue
        j = where[richest[rep[i]]]
        if j == i or len(members[i]) + len(members[j]) > limit:
            continue
        for v in members[i]:
            where[v] = j
        members[j].extend(members.pop(i))
        if j not in rep or rich_degree(rep[j]) < rich_degree(rep[i]):
            rep[j] = rep[i]
        pending.add(j)
    return where


def list_schedule(sizes: Dict[int, int], p: int) -> Dict[int, int]:
    """Alg. 1, assigning clusters to partitions: cluster number -> partition."""
    load = [0] * p
    out = {}
    for c in sorted(sizes, key=lambda c: (-sizes[c], c)):
        t = min(range(p), key=lambda s: (load[s], s))
        out[c] = t
        load[t] += sizes[c]
    return out


def spring(n: int, degree: Sequence[int], edges: Sequence[Tuple[int, int]], p: int, beta: float, tau_vol: int):
    """All three steps.  Returns dict(part, cluster_stream, cluster_merged)."""
    cluster, _, richest = stream_clustering(n, degree, edges, tau_vol)
    merged = merge_clusters(n, degree, cluster, richest, p, beta)
    sizes: Dict[int, int] = {}
    for c in merged:
        sizes[c] = sizes.get(c, 0) + 1
    assign = list_schedule(sizes, p)
    return dict(part=[assign[c] for c in merged], cluster_stream=cluster, cluster_merged=merged)


def partition_graph(n: int, adjacency: Sequence[Sequence[int]], part: Sequence[int], which: int):
    """Edge pass for one partition.  Local ids: owned nodes in ascending global id,
    then the replicas in ascending global id.  Returns (global_id list, n_owned,
    local adjacency lists sorted ascending); a replica's list holds only its
    neighbours owned by this partition."""
    owned = [v for v in range(n) if part[v] == which]
    own = set(owned)
    replicas = sorted({w for v in owned for w in adjacency[v] if w not in own})
    global_id = owned + replicas
    local = {g: i for i, g in enumerate(global_id)}
    rows = []
    for g in global_id:
        if g in own:
            rows.append(sorted(local[w] for w in adjacency[g]))
        else:
            rows.append(sorted(local[w] for w in adjacency[g] if w in own))
    return global_id, len(owned), rows


def replication_factor(n: int, adjacency: Sequence[Sequence[int]], part: Sequence[int], p: int) -> float:
    """Sum over partitions of their node counts, replicas included, over |V|."""
    return sum(len(partition_graph(n, adjacency, part, k)[0]) for k in range(p)) / n
