"""Parser for tests/golden/basis_case.txt (hand-written expected values)."""
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def load_basis_case(storage=np.float32):
    d = None
    lists, queries, expects = {}, {}, []
    with open(os.path.join(HERE, "golden", "basis_case.txt")) as f:
        for line in f:
            t = line.split()
            if not t or t[0].startswith("#"):
                continue
            if t[0] == "d":
                d = int(t[1])
            elif t[0] == "list":
                i, a = t.index("ids"), t.index("a")
                lists[int(t[1])] = ([int(x) for x in t[i + 1:a]], [float(x) for x in t[a + 1:]])
            elif t[0] == "query":
                queries[t[1]] = np.array([float(x) for x in t[2:]], dtype=np.float32)
            elif t[0] == "expect":
                p, i, s = t.index("probes"), t.index("ids"), t.index("scores")
                expects.append(dict(query=t[1], nprobe=int(t[3]), k=int(t[5]),
                                    probes=[int(x) for x in t[p + 1:i]],
                                    ids=[int(x) for x in t[i + 1:s]],
                                    scores=[float(x) for x in t[s + 1:]]))
    nlist = d
    cen = np.eye(d, dtype=np.float32)
    offsets = np.zeros(nlist + 1, dtype=np.int64)
    rows, ids = [], []
    for j in range(nlist):
        lid, a = lists[j]
        offsets[j + 1] = offsets[j] + len(lid)
        for u, av in zip(lid, a):
            v = np.zeros(d, dtype=np.float64)
            v[j] = av
            rows.append(v)
            ids.append(u)
    vec = np.array(rows).astype(storage)
    return dict(d=d, nlist=nlist, centroids=cen, vectors=vec, ids=np.array(ids, dtype=np.int64),
                offsets=offsets, queries=queries, expects=expects)
