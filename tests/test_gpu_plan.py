"""Plan outputs (degrees, transposed structure, permutation) against the oracle: bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from gt_inputs import configs, graphs
from gpu_util import announce, up_i32

pytestmark = pytest.mark.gpu


def _cases():
    out = []
    rows = [[1, 2], [], [0, 1, 2, 3, 4, 5], [3, 3, 3], [], [0, 5]]
    rp = np.cumsum([0] + [len(r) for r in rows]).astype(np.int32)
    ci = np.array([c for r in rows for c in r], dtype=np.int32)
    out.append(("hand6_dups_empty", rp, ci, 6))
    out.append(("empty_graph", np.zeros(1, np.int32), np.zeros(0, np.int32), 0))
    out.append(("no_edges", np.zeros(8, np.int32), np.zeros(0, np.int32), 5))
    # one hub row of 5,000 entries (split into work items) inside a sparse bipartite block
    rng = np.random.default_rng(3)
    s = np.concatenate([rng.integers(0, 9000, 5000), rng.integers(0, 9000, 300)])
    d = np.concatenate([np.full(5000, 7), rng.integers(0, 40, 300)])
    rp, ci = graphs.csr_from_pairs(s, d, 40, 9000)
    out.append(("hub_bipartite", rp, ci, 9000))
    c = configs.tiny()["blocks"][0]
    out.append(("c1_tiny", c["rowptr"], c["colidx"], c["n_src"]))
    c = configs.reddit_like(13)["blocks"][0]          # hubs in both directions, > 1 radix tile
    out.append(("rmat13_deg50", c["rowptr"], c["colidx"], c["n_src"]))
    for b in configs.sage_minibatch(12, 64)["blocks"]:
        out.append(("sage_block_%d" % b["n_dst"], b["rowptr"], b["colidx"], b["n_src"]))
    # around the single-launch sort's capacity of 16,384 entries, source ids of one to four bytes
    # (unsorted rows with repeats: the plan takes any CSR)
    for E, n_src in ((16384, 200), (16384, 70000), (16385, 70000), (9000, 1 << 25), (30000, 300)):
        rng = np.random.default_rng(E + n_src)
        deg = rng.multinomial(E, np.ones(700) / 700)
        rp = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
        ci = rng.integers(0, n_src, E).astype(np.int32)
        out.append(("random_E%d_src%d" % (E, n_src), rp, ci, n_src))
    return out


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c[0])
def test_plan_bit_exact(case):
    from paper_2305_17469_amd import binding as B
    name, rp, ci, n_src = case
    announce("plan", name, "n_dst", rp.size - 1, "n_src", n_src, "E", ci.size)
    g = B.Graph(up_i32(rp), up_i32(ci), n_src)
    assert g.validate() == 0
    din, dout, rpt, cit, perm = [t.cpu().numpy() for t in g.outputs()]
    odin, odout = oracle.degrees(rp, ci, n_src)
    orpt, ocit, operm = oracle.transpose(rp, ci, n_src)
    np.testing.assert_array_equal(din, odin)
    np.testing.assert_array_equal(dout, odout)
    np.testing.assert_array_equal(rpt, orpt)
    np.testing.assert_array_equal(perm, operm)
    np.testing.assert_array_equal(cit, ocit)
    info = g.info()
    deg_t = np.diff(orpt) if n_src else np.zeros(0, int)
    chunk = 512                       # 512 entries per work item, halved while E / chunk < 4096 (floor 64)
    while chunk > 64 and ci.size // chunk < 4096:
        chunk //= 2
    for key, deg in (("fwd", odin), ("bwd", deg_t)):
        split = deg > chunk + chunk // 2
        assert info[key + "_split_rows"] == int(split.sum())
        assert info[key + "_items"] == int((~split).sum() + np.ceil(deg[split] / chunk).sum())


def test_validate_counts_violations():
    from paper_2305_17469_amd import binding as B
    announce("plan validate: bad colidx / rowptr")
    rp = np.array([0, 2, 1, 4], dtype=np.int32)          # one decreasing step
    ci = np.array([0, 9, -1, 2], dtype=np.int32)         # two out-of-range sources (n_src = 3)
    # the plan itself must not be built from corrupt arrays; validate works on a separate,
    # well-formed plan of the same sizes whose borrowed arrays are then overwritten
    good_rp = np.array([0, 1, 2, 4], dtype=np.int32)
    good_ci = np.array([0, 1, 2, 2], dtype=np.int32)
    trp, tci = up_i32(good_rp), up_i32(good_ci)
    g = B.Graph(trp, tci, 3)
    assert g.validate() == 0
    g.rowptr.copy_(torch.from_numpy(rp))
    g.colidx.copy_(torch.from_numpy(ci))
    assert g.validate() == 3
