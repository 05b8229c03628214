"""Pins of the CPU oracle's qgZ path (Sec. 3.3 of the paper: all-to-all based
quantized gradient reduction in two hops with tensor-slice reordering, Eq. 1-2;
Sec. 4.1 Alg. 2 for pipeline stages) against the paper's worked example, the
closed form of Eq. (2), the textbook definition of reduce-scatter, and a
float64-route replay of the reduction order."""
import os

import numpy as np
import pytest

import oracle
from oracle import F16, F32
import ref64


def _golden_orders(golden_dir):
    out = []
    for line in open(os.path.join(golden_dir, "reorder_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, seq = line.split(":")
        X, Y = map(int, head.split())
        out.append((X, Y, list(map(int, seq.split()))))
    return out


# ----------------------------------------------------------------------------
# the index map
# ----------------------------------------------------------------------------

def test_reorder_matches_the_papers_examples(golden_dir):
    rows = _golden_orders(golden_dir)
    assert rows[0][:2] == (2, 2)
    for X, Y, seq in rows:
        got = [oracle.reorder_source_slice(p, X, Y, 1) for p in range(X * Y)]
        assert got == seq, (X, Y)


@pytest.mark.parametrize("X,Y", [(2, 2), (8, 48), (8, 64), (16, 24), (5, 7), (1, 9), (9, 1)])
def test_reorder_is_the_closed_form_of_eq2_and_a_bijection(X, Y):
    T = X * Y
    # Eq. (2) read off directly: Y-long runs 0+j, X+j, 2X+j, ... for j = 0..X-1
    eq2 = [i * X + j for j in range(X) for i in range(Y)]
    got = [oracle.reorder_source_slice(p, X, Y, 1) for p in range(T)]
    assert got == eq2
    assert sorted(got) == list(range(T))
    # scatter form (what Alg. 2 returns) is the inverse permutation
    for pid in range(T):
        assert got[oracle.reorder_mapped_slice(pid, X, Y, 1)] == pid
    # the inverse is the same formula with the roles of X and Y exchanged
    inv = [oracle.reorder_source_slice(p, Y, X, 1) for p in range(T)]
    assert [got[inv[p]] for p in range(T)] == list(range(T))
    if X == 1 or Y == 1:
        assert got == list(range(T))


@pytest.mark.parametrize("X,Y,S", [(2, 2, 2), (8, 48, 3), (4, 3, 5)])
def test_stages_permute_inside_each_stage_only(X, Y, S):
    T = X * Y
    one = [oracle.reorder_source_slice(p, X, Y, 1) for p in range(T)]
    got = [oracle.reorder_source_slice(p, X, Y, S) for p in range(S * T)]
    assert got == [st * T + one[w] for st in range(S) for w in range(T)]
    assert sorted(got) == list(range(S * T))
    for pid in range(S * T):
        assert got[oracle.reorder_mapped_slice(pid, X, Y, S)] == pid
    assert oracle.reorder_source_slice(S * T, X, Y, S) == -1


# ----------------------------------------------------------------------------
# fused reorder + quantize == quantize, then move whole blocks
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("X,Y,S,block,bits", [(2, 2, 1, 32, 4), (8, 6, 1, 64, 4), (4, 3, 2, 32, 8), (8, 48, 1, 32, 4)])
def test_fused_reorder_equals_quantize_then_permute(X, Y, S, block, bits):
    from paper_2306_10209_amd import workloads
    slices = X * Y * S
    L = block * 3
    n = slices * L
    g = workloads.as_bits(workloads.gradients(n, seed=21))
    codes, scales = oracle.qgz_reorder(g, F16, X, Y, S, block, bits)
    pc, ps = oracle.qwz_quantize(g, F16, block, bits)
    cb = L * bits // 8
    order = [oracle.reorder_source_slice(p, X, Y, S) for p in range(slices)]
    assert np.array_equal(codes.reshape(slices, cb), pc.reshape(slices, cb)[order])
    assert np.array_equal(scales.reshape(slices, -1), ps.reshape(slices, -1)[order])


# ----------------------------------------------------------------------------
# two hops == reduce-scatter (exact mode), and the misplacement without reorder
# ----------------------------------------------------------------------------

def _two_hop(grads, X, Y, block, bits, reorder=True, divisor=1.0):
    """Simulate qgZ on W = X*Y ranks held as W host buffers.  grads[r]: float32
    array of rank r = node*X + local.  Returns the W final partitions."""
    W = X * Y
    n = grads[0].size
    L = n // W
    m = n // X
    first = []
    for r in range(W):
        if reorder:
            first.append(oracle.qgz_reorder(grads[r], F32, X, Y, 1, block, bits))
        else:
            first.append(oracle.qwz_quantize(grads[r], F32, block, bits))
    cb, sb = m * bits // 8, m // block
    second = {}
    for node in range(Y):
        for j in range(X):
            # intra-node all-to-all: local GPU j receives group j of every peer k in its node
            cin = [first[node * X + k][0][j * cb:(j + 1) * cb] for k in range(X)]
            sin = [first[node * X + k][1][j * sb:(j + 1) * sb] for k in range(X)]
            second[(node, j)] = oracle.qgz_intra_reduce(cin, sin, m, block, bits)
    cl, sl = L * bits // 8, L // block
    out = []
    for node in range(Y):
        for j in range(X):
            # inter-node all-to-all among GPUs with the same local index: from node i, piece `node`
            cin = [second[(i, j)][0][node * cl:(node + 1) * cl] for i in range(Y)]
            sin = [second[(i, j)][1][node * sl:(node + 1) * sl] for i in range(Y)]
            out.append(oracle.qgz_inter_reduce(cin, sin, L, block, bits, divisor))
    return out


@pytest.mark.parametrize("X,Y", [(2, 2), (4, 3), (8, 2), (3, 5)])
def test_two_hops_with_reorder_are_a_reduce_scatter(X, Y):
    W, block = X * Y, 32
    L = 2 * block
    rng = np.random.default_rng(X * 100 + Y)
    grads = [rng.integers(-50, 50, size=W * L).astype(np.float32) for _ in range(W)]
    total = np.sum(np.stack(grads), axis=0)                 # integers: exact in fp32
    got = _two_hop(grads, X, Y, block, bits=32)
    for r in range(W):
        assert np.array_equal(got[r], total[r * L:(r + 1) * L]), r
    avg = _two_hop(grads, X, Y, block, bits=32, divisor=float(W))
    for r in range(W):
        assert np.array_equal(avg[r], (total[r * L:(r + 1) * L].astype(np.float64) / W).astype(np.float32))


def test_without_reorder_partitions_are_misplaced_as_the_paper_describes():
    """Sec. 3.3.3, 2 machines x 2 GPUs: without the reordering G1 ends with
    partition 3's data and G2 with partition 2's (1-indexed)."""
    X = Y = 2
    W, block, L = 4, 32, 32
    rng = np.random.default_rng(1)
    grads = [rng.integers(-9, 9, size=W * L).astype(np.float32) for _ in range(W)]
    total = np.sum(np.stack(grads), axis=0).reshape(W, L)
    got = _two_hop(grads, X, Y, block, bits=32, reorder=False)
    assert np.array_equal(got[0], total[0]) and np.array_equal(got[3], total[3])
    assert np.array_equal(got[1], total[2]) and np.array_equal(got[2], total[1])
    assert not np.array_equal(total[1], total[2])


# ----------------------------------------------------------------------------
# the reduce stages with quantization: replay of the order by the float64 route
# ----------------------------------------------------------------------------

def _quantized_inputs(K, m, block, bits, seed):
    from paper_2306_10209_amd import workloads
    cs = []
    for k in range(K):
        g = workloads.as_bits(workloads.gradients(m, seed=seed, tensor_id=k))
        cs.append(oracle.qwz_quantize(g, F16, block, bits))
    return [c for c, _ in cs], [s for _, s in cs]


@pytest.mark.parametrize("X,block,bits", [(8, 512, 4), (3, 32, 4), (8, 64, 8), (1, 32, 4)])
def test_intra_reduce_matches_ordered_replay(X, block, bits):
    m = block * 9
    cin, sin = _quantized_inputs(X, m, block, bits, seed=31)
    codes, scales = oracle.qgz_intra_reduce(cin, sin, m, block, bits)
    terms = [ref64.dequant(oracle.unpack_codes(c, m, bits), s, block) for c, s in zip(cin, sin)]
    r = ref64.fold_sum(terms)
    q_ref, s_ref = ref64.quant_blocks(r, block, bits)
    assert np.array_equal(scales.view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(oracle.unpack_codes(codes, m, bits), q_ref)


@pytest.mark.parametrize("Y,block,bits,div", [(48, 512, 4, 384.0), (5, 32, 4, 1.0), (6, 64, 8, 48.0)])
def test_inter_reduce_matches_ordered_replay(Y, block, bits, div):
    m = block * 5
    cin, sin = _quantized_inputs(Y, m, block, bits, seed=32)
    out = oracle.qgz_inter_reduce(cin, sin, m, block, bits, div)
    terms = [ref64.dequant(oracle.unpack_codes(c, m, bits), s, block) for c, s in zip(cin, sin)]
    want = ref64.rn32(ref64.fold_sum(terms) / div)
    assert np.array_equal(out.astype(np.float64), want)


def test_summation_order_is_ascending_peer_index():
    """A case where fp32 addition is not associative: the result must be the
    left-to-right fold over peer index, not any other order."""
    block, m = 32, 32
    vals = [1.0, 2.0 ** -24, 2.0 ** -24, -1.0]            # fold: ((1+e)+e)-1 = 0 ; reversed: 2^-23
    for bits in (32, 8):
        cin, sin = [], []
        for v in vals:
            x = np.zeros(m, dtype=np.float32)
            if bits == 8:                                  # 127*|v| sets the scale to |v| exactly,
                x[0], x[1] = 64.0 * v, 127.0 * abs(v)      # so 64*v is coded as +-64 and decodes exactly
            else:
                x[0] = v
            c, s = oracle.qwz_quantize(x, F32, block, bits)
            cin.append(c)
            sin.append(s)
        if bits == 32:
            out = oracle.qgz_inter_reduce(cin, sin, m, block, bits, 1.0)
            assert out[0] == 0.0
            out = oracle.qgz_inter_reduce(cin[::-1], sin[::-1], m, block, bits, 1.0)
            assert out[0] == np.float32(2.0 ** -23)
            c2, s2 = oracle.qgz_intra_reduce(cin[::-1], sin[::-1], m, block, bits)
            assert c2.view(np.float32)[0] == np.float32(2.0 ** -23)
            c2, s2 = oracle.qgz_intra_reduce(cin, sin, m, block, bits)
            assert c2.view(np.float32)[0] == 0.0
        else:
            # 64, 2^-18, 2^-18, -64: the fold loses both small terms only in this order
            fwd = oracle.qgz_inter_reduce(cin, sin, m, block, bits, 1.0)[0]
            bwd = oracle.qgz_inter_reduce(cin[::-1], sin[::-1], m, block, bits, 1.0)[0]
            assert fwd == 0.0 and bwd == np.float32(2.0 ** -17)


@pytest.mark.parametrize("X,Y", [(4, 3), (8, 2)])
def test_quantized_two_hop_error_is_within_the_step_bound(X, Y):
    """The quantized path's result differs from the exact mean by at most the
    half-steps of the blocks it went through (first hop: one per contributing
    rank; second hop: one per node), divided by W."""
    from paper_2306_10209_amd import workloads
    W, block, bits = X * Y, 32, 4
    L = 2 * block
    n = W * L
    grads16 = [workloads.as_bits(workloads.gradients(n, seed=41, tensor_id=r)) for r in range(W)]
    grads = [ref64.f16_bits_to_f64(g).astype(np.float32) for g in grads16]
    got = _two_hop(grads, X, Y, block, bits, divisor=float(W))
    exact = np.mean(np.stack([g.astype(np.float64) for g in grads]), axis=0)
    # recompute the scales along the path to evaluate the bound
    first = [oracle.qgz_reorder(g, F32, X, Y, 1, block, bits) for g in grads]
    m = n // X
    sb, sl = m // block, L // block
    for node in range(Y):
        for j in range(X):
            r = node * X + j
            bound = np.zeros(L)
            for i in range(Y):          # node i's second-hop block scales for the piece sent to `node`
                cin = [first[i * X + k][0][j * (m // 2):(j + 1) * (m // 2)] for k in range(X)]
                sin = [first[i * X + k][1][j * sb:(j + 1) * sb] for k in range(X)]
                _, s2 = oracle.qgz_intra_reduce(cin, sin, m, block, bits)
                bound += np.repeat(s2[node * sl:(node + 1) * sl].astype(np.float64), block) / 2
                for k in range(X):
                    bound += np.repeat(sin[k][node * sl:(node + 1) * sl].astype(np.float64), block) / 2
            bound = bound / W * (1 + 2.0 ** -12)
            err = np.abs(got[r].astype(np.float64) - exact[r * L:(r + 1) * L])
            assert np.all(err <= bound), (r, float(np.max(err - bound)))
            assert np.max(err) > 0      # it is a lossy path: the bound is not vacuous


def test_fused_stage_traffic_is_one_ninth_of_the_unfused_sequence():
    """Sec. 4.2: fusing dequantize -> reduce -> quantize cuts memory traffic ~9x.
    Per output element with N int4 inputs and 16-bit intermediates the unfused
    sequence moves (0.5N + 2N) + (2N + 2) + (2 + 0.5) bytes, the fused one
    0.5N + 0.5."""
    for N in (2, 8, 16, 48):
        unfused = (0.5 * N + 2 * N) + (2 * N + 2) + (2 + 0.5)
        fused = oracle.codes_nbytes(2 * N, 4) / 2 + oracle.codes_nbytes(2, 4) / 2
        assert unfused / fused == 9.0


def test_qgz_invalid_arguments_are_rejected():
    g = np.zeros(4 * 32, dtype=np.uint16)
    with pytest.raises(oracle.OracleError):
        oracle.qgz_reorder(g, F16, 2, 2, 1, 64, 4)         # slice shorter than a block
    with pytest.raises(oracle.OracleError):
        oracle.qgz_reorder(g, F16, 0, 2, 1, 32, 4)
    c, s = oracle.qwz_quantize(g, F16, 32, 4)
    with pytest.raises(oracle.OracleError):
        oracle.qgz_inter_reduce([c], [s], g.size, 32, 4, 0.0)   # divisor must be positive
