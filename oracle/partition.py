"""TEST INFRASTRUCTURE ONLY - slow reference of the hierarchical EBV vertex-cut partitioner
(Sec. 6) and of the partition statistics (Sec. 6 definitions, Sec. 7 ablation table), in plain
Python with sets, one edge at a time, in the paper's notation. Small graphs only.

Readings (the section leaves them open): edges are processed by ascending sum of end-vertex
degrees (stable) when sort_edges is set - the order of the EBV algorithm the section builds on -
else as listed; the lowest device wins ties; arithmetic in double, terms added left to right;
the master of a vertex is the replica with most of its edges (lowest device on ties), a vertex
without edges lives on device v mod p.
"""


def ebv_partition(n_vertices, edges, p, devices_per_host=1, alpha=1.0, beta=1.0, gamma=0.1, sort_edges=True):
    """edges: list of (u, v), u != v, each undirected edge once -> list of devices, one per edge."""
    E, V = len(edges), n_vertices
    order = list(range(E))
    if sort_edges:
        deg = [0] * V
        for u, v in edges:
            deg[u] += 1
            deg[v] += 1
        order.sort(key=lambda e: deg[edges[e][0]] + deg[edges[e][1]])      # list.sort is stable
    d_rep = [set() for _ in range(V)]
    h_rep = [set() for _ in range(V)]
    e_count = [0] * p
    v_count = [0] * p
    host = [i // devices_per_host for i in range(p)]
    part = [None] * E
    for e in order:
        u, v = edges[e]
        best, best_eva = None, None
        for i in range(p):
            eva = (1.0 - gamma) * float((i not in d_rep[u]) + (i not in d_rep[v]))
            eva = eva + gamma * float((host[i] not in h_rep[u]) + (host[i] not in h_rep[v]))
            eva = eva + alpha * (float(e_count[i]) / (float(E) / p))
            eva = eva + beta * (float(v_count[i]) / (float(V) / p))
            if best is None or eva < best_eva:
                best, best_eva = i, eva
        part[e] = best
        e_count[best] += 1
        for x in (u, v):
            if best not in d_rep[x]:
                d_rep[x].add(best)
                v_count[best] += 1
            h_rep[x].add(host[best])
    return part


def cut_statistics(n_vertices, edges, part, p, devices_per_host=1):
    """-> dict(replication_factor, edge_imbalance, vertex_imbalance, max_inner, max_outer, replicas_total, master)"""
    V, E = n_vertices, len(edges)
    V_i = [set() for _ in range(p)]
    E_i = [0] * p
    inc = [[0] * p for _ in range(V)]
    for (u, v), i in zip(edges, part):
        E_i[i] += 1
        V_i[i].update((u, v))
        inc[u][i] += 1
        inc[v][i] += 1
    master = []
    for v in range(V):
        if any(inc[v]):
            master.append(max(range(p), key=lambda i: (inc[v][i], -i)))
        else:
            master.append(v % p)
            V_i[v % p].add(v)
    host = [i // devices_per_host for i in range(p)]
    inner, outer = [0] * p, [0] * p
    for i in range(p):
        for v in V_i[i]:
            m = master[v]
            if m == i:
                continue
            tgt = inner if host[i] == host[m] else outer
            tgt[i] += 1      # gather message, mirror -> master
            tgt[m] += 1      # scatter message, master -> mirror
    replicas = sum(len(s) for s in V_i)
    return dict(replication_factor=replicas / V,
                edge_imbalance=(max(E_i) / (E / p)) if E else 1.0,
                vertex_imbalance=max(len(s) for s in V_i) / (replicas / p),
                max_inner=max(inner), max_outer=max(outer), replicas_total=replicas, master=master)
