"""Host-side rows next to the hot path: partition into sequential sub-graphs (Appendix B), gain
formulas (Sec. 2.3.2, 2.3.3) and the Prefix / Random baselines (Sec. 3.1).  The library's C++
(dominator-tree formulation) is compared with a brute-force Python statement of what a sequential
sub-graph is (take a vertex out; if the sink is cut off from the start, the vertex closes a group), and
both are pinned to the partition the paper shows for a Llama-3 layer."""
import numpy as np
import pytest

import paper_2505_13060_amd as amp
from oracle import partition as orc


def llama_graph(n_blocks, residual=False):
    """Vertices and edges of n decoder blocks + LM head.  Returns (names, edges, quantizable)."""
    names, edges = ["embed"], []
    prev = 0

    def add(name, preds):
        names.append(name)
        v = len(names) - 1
        for p in preds:
            edges.append((p, v))
        return v

    for b in range(n_blocks):
        t = "b%d." % b
        n1 = add(t + "norm1", [prev])
        q, k, v = add(t + "q_proj", [n1]), add(t + "k_proj", [n1]), add(t + "v_proj", [n1])
        qk = add(t + "qk_matmul", [q, k])
        sm = add(t + "softmax", [qk])
        av = add(t + "av_matmul", [sm, v])
        o = add(t + "o_proj", [av])
        h = add(t + "add1", [o, prev]) if residual else o
        n2 = add(t + "norm2", [h])
        g, u = add(t + "gate_proj", [n2]), add(t + "up_proj", [n2])
        act = add(t + "act", [g])
        mul = add(t + "mul", [act, u])
        d = add(t + "down_proj", [mul])
        prev = add(t + "add2", [d, h]) if residual else d
    fn = add("final_norm", [prev])
    add("lm_head", [fn])
    quant = [int(n.endswith("_proj") or n.endswith("_matmul") or n == "lm_head") for n in names]
    return names, edges, quant


def groups_from(group_of, n_groups):
    out = [[] for _ in range(n_groups)]
    for v, g in enumerate(group_of):
        if g >= 0:
            out[g].append(v)
    return out


def test_llama_layer_partition_matches_the_papers_figure():
    names, edges, quant = llama_graph(2)
    group_of, ng = amp.amp_partition_sequential(len(names), edges, quant)
    got = [sorted(names[v].split(".")[-1] for v in g) for g in groups_from(group_of, ng)]
    block = [sorted(["q_proj", "k_proj", "v_proj", "qk_matmul", "av_matmul"]), ["o_proj"],
             sorted(["gate_proj", "up_proj"]), ["down_proj"]]
    assert got == block + block + [["lm_head"]]
    want = orc.partition_sequential(len(names), edges, quant)
    assert groups_from(group_of, ng) == want
    # five quantisable ops in the attention sub-graph -> 2^5 = 32 configurations for F = 2
    assert len(got[0]) == 5


def test_residual_edges_merge_the_block_as_single_entry_single_exit_demands():
    names, edges, quant = llama_graph(1, residual=True)
    group_of, ng = amp.amp_partition_sequential(len(names), edges, quant)
    got = [sorted(names[v].split(".")[-1] for v in g) for g in groups_from(group_of, ng)]
    assert got == [sorted(["q_proj", "k_proj", "v_proj", "qk_matmul", "av_matmul", "o_proj"]),
                   sorted(["gate_proj", "up_proj", "down_proj"]), ["lm_head"]]
    assert groups_from(group_of, ng) == orc.partition_sequential(len(names), edges, quant)


def test_sequential_model_gives_one_group_per_layer():
    n = 9
    edges = [(i, i + 1) for i in range(n - 1)]
    group_of, ng = amp.amp_partition_sequential(n, edges)
    assert ng == n - 1 and list(group_of) == [-1] + list(range(n - 1))


def random_dag(rng, n):
    edges = set()
    for v in range(1, n):
        edges.add((int(rng.integers(max(0, v - 4), v)), v))
    for v in range(n - 1):
        if not any(a == v for a, _ in edges):
            edges.add((v, int(rng.integers(v + 1, min(n, v + 5)))))
    for _ in range(int(rng.integers(0, n))):
        a = int(rng.integers(0, n - 1))
        edges.add((a, int(rng.integers(a + 1, min(n, a + 6)))))
    return sorted(edges)


@pytest.mark.parametrize("seed", range(60))
def test_partition_matches_the_brute_force_definition_on_random_dags(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 40))
    edges = random_dag(rng, n)
    quant = (rng.random(n) < 0.7).astype(np.uint8) if seed % 3 else None
    group_of, ng = amp.amp_partition_sequential(n, edges, quant)
    assert groups_from(group_of, ng) == orc.partition_sequential(n, edges, quant)
    # every quantisable vertex except the start is in exactly one group
    for v in range(1, n):
        assert (group_of[v] >= 0) == (quant is None or bool(quant[v]))
    assert group_of[0] == -1


def test_partition_rejects_bad_graphs():
    for n, edges in [(3, [(0, 1), (1, 2), (2, 0)]),           # cycle
                     (3, [(0, 2), (1, 2)]),                   # two sources
                     (3, [(0, 1), (0, 2)]),                   # two sinks
                     (2, [(0, 5)])]:                          # vertex out of range
        with pytest.raises(amp.AmpError) as ei:
            amp.amp_partition_sequential(n, edges)
        assert ei.value.status == amp.ERR_INVALID_ARG


def test_gain_formulas():
    # Sec. 2.3.2: N C K delta (linear), N C^2 delta (BGEMM); Sec. 2.3.3: C K delta_M, 0 for BGEMM
    assert amp.amp_time_gain_macs(0, 40, 4096, 11008, 0.5) == 40 * 4096 * 11008 * 0.5
    assert amp.amp_time_gain_macs(1, 40, 128, 999, 0.5) == 40 * 128 * 128 * 0.5
    assert amp.amp_memory_gain(0, 4096, 11008, 1.0) == 4096 * 11008
    assert amp.amp_memory_gain(1, 4096, 11008, 1.0) == 0.0


def tables(rng, J, F=2):
    n_choices = np.full(J, F, dtype=np.int32)
    gain = np.zeros((J, F))
    mse = np.zeros((J, F))
    gain[:, 1:] = rng.uniform(0.5, 3.0, (J, F - 1))
    mse[:, 1:] = np.exp(rng.normal(0, 1.5, (J, F - 1)))
    return n_choices, gain.reshape(-1), mse.reshape(-1)


@pytest.mark.parametrize("seed", range(20))
def test_prefix_and_random_baselines(seed):
    rng = np.random.default_rng(seed)
    J = int(rng.integers(1, 30))
    n_choices, gain, mse = tables(rng, J, F=2 + seed % 2)
    budget = float(rng.uniform(0, 0.5) * mse.reshape(J, -1).max(axis=1).sum())
    # Prefix
    choice, g, d = amp.amp_select_ordered(n_choices, gain, mse, budget)
    want = orc.select_ordered(list(n_choices), list(gain), list(mse), budget)
    assert list(choice) == want[0] and g == pytest.approx(want[1], rel=1e-12) and d == pytest.approx(want[2], rel=1e-12)
    assert d <= budget
    k = int(np.count_nonzero(choice))
    assert np.all(choice[:k] != 0) and np.all(choice[k:] == 0)      # a prefix of the layers
    # Random
    order = rng.permutation(J).astype(np.int32)
    choice_r, g_r, d_r = amp.amp_select_ordered(n_choices, gain, mse, budget, order)
    want = orc.select_ordered(list(n_choices), list(gain), list(mse), budget, list(order))
    assert list(choice_r) == want[0] and d_r <= budget
    # the IP solution is at least as good as both under the same bound (Sec. 3.3)
    _, g_ip, d_ip = amp.amp_select_subgraphs(n_choices, gain, mse, budget)
    assert d_ip <= budget and g_ip >= g - 1e-12 and g_ip >= g_r - 1e-12


def test_select_ordered_errors():
    n_choices = np.array([2, 2], dtype=np.int32)
    gain = np.array([0.0, 1.0, 0.0, 1.0])
    mse = np.array([0.0, 1.0, 0.0, 1.0])
    with pytest.raises(amp.AmpError):
        amp.amp_select_ordered(n_choices, gain, mse, 1.0, np.array([0, 0], dtype=np.int32))   # not a permutation
    mse0 = np.array([2.0, 1.0, 0.0, 1.0])
    with pytest.raises(amp.AmpError) as ei:
        amp.amp_select_ordered(n_choices, gain, mse0, 1.0)       # even the high-precision columns exceed the budget
    assert ei.value.status == amp.ERR_INFEASIBLE
