"""TEST INFRASTRUCTURE -- brute-force oracle for the intra-stream schedule (integers only).

Section 3.1 of the paper: strongly connected components are found; a component that is
not a singleton, or a singleton with a self-loop, becomes one "recurrent node"; the rest
is a DAG whose nodes are worked on for all frames at once in topological order; inside a
recurrent node each time step computes the delayed connections first and then the
remaining (acyclic) part in topological order.

This oracle does not use Tarjan's algorithm (the product's analyser does): it computes
the transitive closure by Warshall's algorithm and reads the components off mutual
reachability.  Because several topological orders / component numberings are valid, the
exported schedule is canonical, defined by longest-path levels:

  comp_level(C)   0 if no edge enters C from another component, else 1 + max over the
                  components such edges come from (delays ignored)
  node_comp[v]    components numbered 0.. by increasing (comp_level, smallest node id)
  comp_recurrent  1 iff the component has more than one node or an edge with src = dst
  node_level[v]   level inside one time step: for a node of a recurrent component,
                  0 if it has no delay-0 in-edge from the same component, else 1 + max
                  node_level over the sources of such edges; 0 for all other nodes
  edge_class[m]   0 BATCHED       source and destination in different components
                  1 STEP_DELAYED  same component, delay >= 1
                  2 STEP_DELAY0   same component, delay == 0
"""
from __future__ import annotations

BATCHED, STEP_DELAYED, STEP_DELAY0 = 0, 1, 2


def schedule(nodes, edges):
    K = len(nodes)
    reach = [[False] * K for _ in range(K)]
    for e in edges:
        reach[e["src"]][e["dst"]] = True
    for via in range(K):
        for a in range(K):
            if reach[a][via]:
                ra, rv = reach[a], reach[via]
                for b in range(K):
                    if rv[b]:
                        ra[b] = True
    # components = classes of mutual reachability, keyed by their smallest node id
    rep = list(range(K))
    for a in range(K):
        for b in range(a):
            if reach[a][b] and reach[b][a]:
                rep[a] = rep[b]
                break
    members = {}
    for v in range(K):
        members.setdefault(rep[v], []).append(v)
    reps = sorted(members)
    recurrent = {r: (len(members[r]) > 1) for r in reps}
    for e in edges:
        if e["src"] == e["dst"]:
            recurrent[rep[e["src"]]] = True
    # longest-path level of each component in the condensation
    level = {r: None for r in reps}

    def comp_level(r):
        if level[r] is None:
            best = 0
            for e in edges:
                if rep[e["dst"]] == r and rep[e["src"]] != r:
                    best = max(best, 1 + comp_level(rep[e["src"]]))
            level[r] = best
        return level[r]

    for r in reps:
        comp_level(r)
    numbering = {r: i for i, r in enumerate(sorted(reps, key=lambda r: (level[r], r)))}
    node_comp = [numbering[rep[v]] for v in range(K)]
    node_comp_level = [level[rep[v]] for v in range(K)]
    node_recurrent = [int(recurrent[rep[v]]) for v in range(K)]
    # level inside a time step
    nlevel = [None] * K

    def node_level(v):
        if nlevel[v] is None:
            nlevel[v] = -1          # cycle guard
            best = 0
            if recurrent[rep[v]]:
                for e in edges:
                    if e["dst"] == v and e["delay"] == 0 and rep[e["src"]] == rep[v]:
                        lv = node_level(e["src"])
                        if lv < 0:
                            raise ValueError("delay-0 edges form a cycle")
                        best = max(best, 1 + lv)
            nlevel[v] = best
        return nlevel[v]

    for v in range(K):
        node_level(v)
    edge_class = []
    for e in edges:
        if rep[e["src"]] != rep[e["dst"]]:
            edge_class.append(BATCHED)
        elif e["delay"] >= 1:
            edge_class.append(STEP_DELAYED)
        else:
            edge_class.append(STEP_DELAY0)
    return dict(node_comp=node_comp, node_level=nlevel, comp_level=node_comp_level,
                comp_recurrent=node_recurrent, edge_class=edge_class, n_comps=len(reps))
