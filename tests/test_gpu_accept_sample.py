"""GPU parity (bit-exact) of tree_accept_sample against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import accept_sample as A
from oracle import pack_accept as PA
from paper_2604_09731_amd import binding as B
from paper_2604_09731_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return B.SmartTree(0)


def _dev(a, dtype=None):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype)).to("cuda")


def _case(seed, sizes, V, peaked=True):
    """Trees whose children propose distinct likely tokens, and a target that agrees with the drafts about
    half of the time (so walks of every length occur)."""
    rng = np.random.default_rng(seed)
    trees = [W.random_tree(n, rng, str(rng.choice(["random", "chain", "star"]))) for n in sizes]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate(trees).astype(np.int32)
    N = int(cu[-1])
    token = rng.integers(0, V, N).astype(np.int32)
    prob = rng.random((N, V)).astype(np.float32) ** (8 if peaked else 1)
    for b in range(len(sizes)):                      # move mass onto the tokens the children of each node propose
        base = int(cu[b])
        for i in range(int(sizes[b])):
            kids = [c for c in range(i + 1, int(sizes[b])) if parent[base + c] == i]
            for c in kids:
                prob[base + i, token[base + c]] += rng.random() * prob[base + i].sum() / max(1, len(kids))
    prob /= prob.sum(1, keepdims=True)
    return cu, parent, token, prob.astype(np.float32)


@pytest.mark.parametrize("V,sizes", [(5, [1, 2, 9, 40]), (64, [128, 3, 17]), (1000, [33, 64, 65, 1, 12]),
                                     (4099, [20, 45]), (32000, [24, 7])])
def test_bit_exact_against_the_oracle(lib, V, sizes):
    import torch
    cu, parent, token, prob = _case(V, sizes, V)
    d = (_dev(cu), _dev(parent), _dev(token), _dev(prob))
    for seed, step, max_depth in ((1, 0, 8), (2 ** 40 + 5, 2 ** 33 + 1, 3), (7, 12345, 0)):
        al, path, bonus = lib.tree_accept_sample(*d, max_depth, seed, step)
        torch.cuda.synchronize()
        o_al, o_path, o_bonus = A.accept_sample(cu, parent, token, prob, seed, step, max_depth)
        assert al.cpu().numpy().tolist() == o_al
        assert path.cpu().numpy().tolist() == o_path
        assert bonus.cpu().numpy().tolist() == o_bonus
    lens = set()
    for step in range(12):                           # walks of several lengths were really taken
        al, _, _ = lib.tree_accept_sample(*d, 8, 3, step)
        lens |= set(al.cpu().numpy().tolist())
    assert len(lens) >= 2 or max(sizes) < 3


def test_strided_rows_duplicates_and_out_of_range_tokens(lib):
    import torch
    V = 300
    cu, parent, token, prob = _case(77, [30, 30, 6], V)
    token[3], token[4] = V + 5, -2                                  # proposals outside the vocabulary are skipped
    sib = [c for c in range(1, 30) if parent[c] == 0]
    if len(sib) >= 2:
        token[sib[1]] = token[sib[0]]                               # a duplicate proposal
    wide = torch.full((prob.shape[0], V + 37), float("nan"), dtype=torch.float32, device="cuda")
    wide[:, :V] = _dev(prob)
    view = wide[:, :V]                                              # row stride 337: the unaligned path
    for step in range(6):
        al, path, bonus = lib.tree_accept_sample(_dev(cu), _dev(parent), _dev(token), view, 6, 11, step)
        torch.cuda.synchronize()
        o = A.accept_sample(cu, parent, token, prob, 11, step, 6)
        assert (al.cpu().numpy().tolist(), path.cpu().numpy().tolist(), bonus.cpu().numpy().tolist()) == o


def test_point_mass_target_equals_the_greedy_walk_and_edge_cases(lib):
    import torch
    rng = np.random.default_rng(5)
    sizes = [1, 7, 30, 64, 128]
    trees = [W.random_tree(n, rng, "random") for n in sizes]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate(trees).astype(np.int32)
    N, V = int(cu[-1]), 6
    token = rng.integers(0, V, N).astype(np.int32)
    target_next = rng.integers(0, V, N).astype(np.int32)
    prob = np.zeros((N, V), np.float32)
    prob[np.arange(N), target_next] = 1.0
    d = (_dev(cu), _dev(parent), _dev(token))
    al, path, bonus = lib.tree_accept_sample(*d, _dev(prob), 7, 99, 3)
    g_al, g_path, g_bonus = lib.tree_accept(*d, _dev(target_next), 7)
    torch.cuda.synchronize()
    assert torch.equal(al, g_al) and torch.equal(path, g_path) and torch.equal(bonus, g_bonus)
    assert al.cpu().numpy().tolist() == PA.accept(cu, parent, token, target_next, 7)[0]
    # no mass anywhere: nothing accepted, no bonus; offsets outside the arrays: flagged
    zero = torch.zeros((N, V), dtype=torch.float32, device="cuda")
    al, path, bonus = lib.tree_accept_sample(*d, zero, 7, 1, 1)
    assert al.cpu().numpy().tolist() == [0] * 5 and bonus.cpu().numpy().tolist() == [-1] * 5
    bad_cu = cu.copy()
    bad_cu[-1] = N + 50
    al, path, bonus = lib.tree_accept_sample(_dev(bad_cu), d[1], d[2], _dev(prob), 7, 1, 1)
    assert al.cpu().numpy().tolist()[-1] == -1 and bonus.cpu().numpy().tolist()[-1] == -1
    assert al.cpu().numpy().tolist()[:4] == g_al.cpu().numpy().tolist()[:4]


def test_emitted_tokens_follow_the_target_distribution(lib):
    """20000 sequences with the same two-proposal tree and target, one launch: the first emitted token's
    histogram against the integer weights (chi-square, 11 degrees of freedom)."""
    import torch
    rng = np.random.default_rng(0)
    V, nseq = 12, 20000
    p = rng.dirichlet(np.ones(V)).astype(np.float32)
    cu = (np.arange(nseq + 1) * 3).astype(np.int32)
    parent = np.tile(np.array([-1, 0, 0], np.int32), nseq)
    tok3 = np.array([0, int(np.argmax(p)), int(np.argmin(p))], np.int32)
    token = np.tile(tok3, nseq)
    prob = torch.from_numpy(p).cuda().repeat(3 * nseq, 1)
    al, path, bonus = lib.tree_accept_sample(_dev(cu), _dev(parent), _dev(token), prob, 1, 42, 0)
    torch.cuda.synchronize()
    al, path, bonus = al.cpu().numpy(), path.cpu().numpy(), bonus.cpu().numpy()
    first = np.where(al >= 1, tok3[np.maximum(path[:, 1], 0)], bonus)
    hist = np.bincount(first, minlength=V).astype(np.float64)
    w = np.array(A.weights(p), np.float64)
    expect = w / w.sum() * nseq
    chi2 = float(((hist - expect) ** 2 / expect).sum())
    assert chi2 < 40.0, chi2
    # and a sample of the sequences is bit-identical to the oracle (the sequence index feeds the generator)
    o = A.accept_sample(cu[:41], parent[:120], token[:120], np.tile(p, (120, 1)), 42, 0, 1)
    assert al[:40].tolist() == o[0] and bonus[:40].tolist() == o[2]
