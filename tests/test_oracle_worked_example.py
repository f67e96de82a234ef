"""The paper's worked example (two KV heads, block size 2, 5 and 2 KVs): pinned
by structure, from tests/golden/worked_example_two_heads.txt."""
import os

import numpy as np

from oracle import kvc_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def load_fixture():
    fx = {"metrics": {}}
    with open(os.path.join(HERE, "golden", "worked_example_two_heads.txt")) as f:
        for line in f:
            t = line.split()
            if not t or t[0].startswith("#"):
                continue
            if t[0] == "block_size":
                fx["b"] = int(t[1])
            elif t[0] == "head":
                fx["metrics"][int(t[1])] = [float(x) for x in t[3:]]
            else:
                fx[t[0]] = {t[i]: int(t[i + 1]) for i in range(1, len(t), 2)}
    return fx


def build(fx):
    b = fx["b"]
    lens = np.array([len(fx["metrics"][0]), len(fx["metrics"][1])])
    nb = -(-lens // b)
    N = int(nb.sum()); maxb = int(nb.max())
    table = -np.ones((2, maxb), dtype=np.int64)
    M = np.zeros((N, b)); p = 0
    K = np.zeros((N, b, 1)); pos = np.zeros((N, b))
    for h in range(2):
        for u in range(nb[h]):
            table[h, u] = p; p += 1
        for j, m in enumerate(fx["metrics"][h]):
            M[table[h, j // b], j % b] = m
            K[table[h, j // b], j % b] = 100 * h + j
            pos[table[h, j // b], j % b] = j
    return O.State(1, 1, 2, 1, 1, b, N, maxb, K, K.copy(), M, pos, table, lens,
                   np.zeros(N, dtype=np.uint8))


def test_two_evictions_come_from_head_zero_third_takes_the_lone_block():
    fx = load_fixture()
    st = build(fx)
    key, _ = O.block_keys(st)
    flag, count, sel = O.evict_select(st, key, [2], protect_tail_blocks=0)
    assert sel[0] == 2
    assert count[0] == fx["evict2"]["head0_blocks"] and count[1] == fx["evict2"]["head1_blocks"]
    flag3, count3, sel3 = O.evict_select(st, key, [3], protect_tail_blocks=0)
    assert sel3[0] == 3
    assert count3[0] == fx["evict3"]["head0_blocks"] and count3[1] == fx["evict3"]["head1_blocks"]
    # with the default protection a head keeps at least its last block
    _, countp, selp = O.evict_select(st, key, [3], protect_tail_blocks=1)
    assert selp[0] == 2 and countp[1] == 0
    freed = O.compact(st, flag, count)
    assert freed == 2
    assert st.lens()[0] == fx["after2"]["head0_len"] and st.lens()[1] == fx["after2"]["head1_len"]
    # the survivor of head 0 is its fifth KV (metric 1.90), now in the first slot
    n, o = O.slots_of(st, 0)
    assert st.metric[n[0], o[0]] == 1.90 and st.k_cache[n[0], o[0], 0] == 4
