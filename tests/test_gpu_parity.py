"""GPU parity: every entry point of the C-ABI library, called through the ctypes
binding, against the CPU oracle on the same seeded inputs.  Integer codes, fp32
scales, 16-bit decodes and fp32 reduced gradients must be bit-identical."""
import numpy as np
import pytest
import torch

import oracle
from paper_2306_10209_amd import binding as zpp
from paper_2306_10209_amd import diagnostics
from paper_2306_10209_amd import workloads

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TORCH_DT = {oracle.F16: torch.float16, oracle.BF16: torch.bfloat16, oracle.F32: torch.float32}


def host_bits(t):
    return workloads.as_bits(t)


def make_input(n, dtype, kind, seed):
    tdt = TORCH_DT[dtype]
    if kind == "weights":
        return workloads.weights(n, seed=seed, dtype=tdt)
    return workloads.gradients(n, seed=seed, dtype=tdt)


def guarded(nbytes_or_numel, dtype):
    """Device buffer with 64 guard elements on both sides, filled with a pattern."""
    pad = 64
    fill = {torch.uint8: 0xA5, torch.float32: -123.25, torch.float16: -77.5, torch.bfloat16: -77.5}[dtype]
    full = torch.full((nbytes_or_numel + 2 * pad,), fill, dtype=dtype, device=DEV)
    return full, full[pad:pad + nbytes_or_numel]


def assert_guards_intact(full, n, dtype):
    pad = 64
    fill = {torch.uint8: 0xA5, torch.float32: -123.25, torch.float16: -77.5, torch.bfloat16: -77.5}[dtype]
    ref = torch.full((pad,), fill, dtype=dtype, device=DEV)
    assert torch.equal(full[:pad], ref) and torch.equal(full[pad + n:], ref), "write outside the output"


def eq_bytes(dev_tensor, host_array):
    got = dev_tensor.detach().cpu().contiguous()
    if got.dtype in (torch.float16, torch.bfloat16):
        got = got.view(torch.int16)
    got = got.numpy().view(np.uint8).reshape(-1)
    want = np.ascontiguousarray(host_array).view(np.uint8).reshape(-1)
    if got.size != want.size:
        return False
    return np.array_equal(got, want)


# ----------------------------------------------------------------------------
# qwZ
# ----------------------------------------------------------------------------

QWZ_CASES = [
    # dtype, bits, block, blocks (odd counts: several tiles and a ragged tail)
    (oracle.F16, 8, 256, 4096),       # the small round-trip configuration: 4096 x 256 fp16
    (oracle.BF16, 8, 2048, 77),
    (oracle.F16, 4, 512, 133),
    (oracle.F16, 8, 32, 1001),
    (oracle.BF16, 4, 64, 517),
    (oracle.F16, 8, 128, 333),
    (oracle.BF16, 8, 1024, 35),
    (oracle.F16, 4, 4096, 13),
    (oracle.F16, 8, 96, 301),         # not a power of two: generic path
    (oracle.BF16, 4, 3072, 7),
    (oracle.F32, 8, 256, 65),
    (oracle.F32, 4, 2048, 9),
    (oracle.F16, 8, 2048, 1),
    (oracle.F16, 4, 32, 1),
    (oracle.BF16, 8, 4064, 19),       # one wave per block, 8 rounds, the last one 60 lanes wide
    (oracle.F16, 4, 2080, 23),        # 5 rounds, the last one 4 lanes wide
    (oracle.F32, 8, 1056, 11),
    (oracle.F16, 4, 4032, 5),
]


@pytest.mark.parametrize("dtype,bits,block,blocks", QWZ_CASES)
def test_qwz_round_trip_bit_exact(dtype, bits, block, blocks):
    n = block * blocks
    kind = "weights" if bits == 8 else "grads"
    x = make_input(n, dtype, kind, seed=block + bits)
    xb = host_bits(x)
    want_codes, want_scales = oracle.qwz_quantize(xb, dtype, block, bits)

    cfull, codes = guarded(n * bits // 8, torch.uint8)
    sfull, scales = guarded(n // block, torch.float32)
    zpp.qwz_quantize(x.to(DEV), block, bits, codes=codes, scales=scales)
    torch.cuda.synchronize()
    assert eq_bytes(scales, want_scales), "scales differ"
    assert eq_bytes(codes, want_codes), "codes differ"
    assert_guards_intact(cfull, n * bits // 8, torch.uint8)
    assert_guards_intact(sfull, n // block, torch.float32)

    for odt in (dtype, oracle.F32):
        want_y = oracle.qwz_dequantize(want_codes, want_scales, n, block, bits, odt)
        yfull, y = guarded(n, TORCH_DT[odt])
        zpp.qwz_dequantize(codes, scales, n, block, bits, out=y)
        torch.cuda.synchronize()
        assert eq_bytes(y, want_y), f"decode to dtype {odt} differs"
        assert_guards_intact(yfull, n, TORCH_DT[odt])


@pytest.mark.parametrize("dtype,bits,block,blocks", [(oracle.BF16, 8, 2048, 16411), (oracle.F16, 8, 256, 270001),
                                                      (oracle.F16, 4, 512, 131075)])
def test_qwz_round_trip_large_grid(dtype, bits, block, blocks):
    """Large enough that the kernels remap workgroups over the XCDs (grids of more
    than 8192 groups), with a ragged last tile; still element by element."""
    n = block * blocks
    x = make_input(n, dtype, "weights", seed=blocks)
    want_codes, want_scales = oracle.qwz_quantize(host_bits(x), dtype, block, bits)
    cfull, codes = guarded(n * bits // 8, torch.uint8)
    sfull, scales = guarded(n // block, torch.float32)
    zpp.qwz_quantize(x.to(DEV), block, bits, codes=codes, scales=scales)
    yfull, y = guarded(n, TORCH_DT[dtype])
    zpp.qwz_dequantize(codes, scales, n, block, bits, out=y)
    torch.cuda.synchronize()
    assert eq_bytes(scales, want_scales) and eq_bytes(codes, want_codes)
    assert eq_bytes(y, oracle.qwz_dequantize(want_codes, want_scales, n, block, bits, dtype))
    assert_guards_intact(cfull, n * bits // 8, torch.uint8)
    assert_guards_intact(sfull, n // block, torch.float32)
    assert_guards_intact(yfull, n, TORCH_DT[dtype])


def test_qwz_shards_written_at_offsets_equal_whole_tensor():
    """The simulated all-gather: P ranks quantize their shard straight into their
    slot of the gather buffer; the result is the whole tensor's quantization."""
    P, block, bits = 8, 2048, 8
    n = P * block * 11
    x = workloads.weights(n, seed=3, dtype=torch.bfloat16)
    want_codes, want_scales = oracle.qwz_quantize(host_bits(x), oracle.BF16, block, bits)
    xd = x.to(DEV)
    codes = torch.zeros(n, dtype=torch.uint8, device=DEV)
    scales = torch.zeros(n // block, dtype=torch.float32, device=DEV)
    sh, shb = n // P, n // P // block
    for r in range(P):
        zpp.qwz_quantize(xd[r * sh:(r + 1) * sh], block, bits, codes=codes[r * sh:(r + 1) * sh],
                         scales=scales[r * shb:(r + 1) * shb])
    y = zpp.qwz_dequantize(codes, scales, n, block, bits, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert eq_bytes(codes, want_codes) and eq_bytes(scales, want_scales)
    assert eq_bytes(y, oracle.qwz_dequantize(want_codes, want_scales, n, block, bits, oracle.BF16))


@pytest.mark.parametrize("bits", [8, 4])
def test_qwz_special_blocks(bits):
    """All-zero, negative-zero, tiny, threshold, largest-fp16, subnormal and
    exact-tie blocks."""
    block = 256
    qmax = (1 << (bits - 1)) - 1
    rows = []
    rows.append(np.zeros(block, dtype=np.float32))
    rows.append(np.full(block, -0.0, dtype=np.float32))
    r = np.zeros(block, dtype=np.float32); r[3] = 2.0 ** -101; rows.append(r)
    r = np.zeros(block, dtype=np.float32); r[0] = 2.0 ** -100; r[1] = -2.0 ** -101; rows.append(r)
    rows.append(np.linspace(-3e38, 3e38, block).astype(np.float32))
    rows.append((np.arange(block) - 31.5).astype(np.float32) * np.float32(1e-42))      # fp32 subnormals
    r = np.zeros(block, dtype=np.float32); r[0] = qmax * 4.0                              # exact ties
    r[1:2 * qmax + 1] = (np.arange(-qmax, qmax) + 0.5) * 4.0
    rows.append(r)
    x32 = np.concatenate(rows)
    codes_w, scales_w = oracle.qwz_quantize(x32, oracle.F32, block, bits)
    codes, scales = zpp.qwz_quantize(torch.from_numpy(x32).to(DEV), block, bits)
    y = zpp.qwz_dequantize(codes, scales, x32.size, block, bits, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert eq_bytes(scales, scales_w) and eq_bytes(codes, codes_w)
    assert eq_bytes(y, oracle.qwz_dequantize(codes_w, scales_w, x32.size, block, bits, oracle.F32))

    # fp16: largest finite values and subnormals
    block = 64
    h = np.zeros(4 * block, dtype=np.float16)
    h[0], h[1], h[2] = 65504.0, -65504.0, 1.0
    h[block:2 * block] = np.arange(block).astype(np.float16) * np.float16(2.0 ** -24)
    h[2 * block + 5] = np.float16(2.0 ** -24)
    hb = h.view(np.uint16)
    cw, sw = oracle.qwz_quantize(hb, oracle.F16, block, bits)
    c, s = zpp.qwz_quantize(torch.from_numpy(h).to(DEV), block, bits)
    y = zpp.qwz_dequantize(c, s, h.size, block, bits, out_dtype=torch.float16)
    torch.cuda.synchronize()
    assert eq_bytes(s, sw) and eq_bytes(c, cw)
    assert eq_bytes(y, oracle.qwz_dequantize(cw, sw, h.size, block, bits, oracle.F16))


def test_decode_rounds_to_nearest_even_in_16_bits():
    """Every int8 code against scales chosen so that products fall between
    16-bit neighbours, including exact ties and the subnormal range."""
    block = 256
    codes_np = np.resize(np.arange(-127, 128, dtype=np.int8), block).view(np.uint8)
    scales_list = [1.0, 1.0 / 3, 2.0 ** -14 / 127, 2.0 ** -24, 3 * 2.0 ** -26, 65504.0 / 127, 2.0 ** -120,
                   1.0009765625, 0.007874016]
    nb = len(scales_list)
    codes = np.tile(codes_np, nb)
    scales = np.array(scales_list, dtype=np.float32)
    cd = torch.from_numpy(codes).to(DEV)
    sd = torch.from_numpy(scales).to(DEV)
    for odt in (oracle.F16, oracle.BF16, oracle.F32):
        y = zpp.qwz_dequantize(cd, sd, block * nb, block, 8, out_dtype=TORCH_DT[odt])
        torch.cuda.synchronize()
        assert eq_bytes(y, oracle.qwz_dequantize(codes, scales, block * nb, block, 8, odt)), odt


# ----------------------------------------------------------------------------
# qgZ: reorder
# ----------------------------------------------------------------------------

REORDER_CASES = [
    # X, Y, S, block, bits, blocks per slice
    (2, 2, 1, 32, 4, 3),
    (8, 6, 1, 512, 4, 5),
    (8, 48, 1, 512, 4, 1),
    (8, 64, 1, 512, 4, 2),
    (4, 3, 2, 64, 8, 9),
    (3, 5, 3, 96, 4, 4),
    (8, 2, 1, 2048, 4, 3),
    (1, 7, 1, 256, 4, 5),
    (16, 1, 2, 128, 8, 3),
    (8, 6, 1, 512, 4, 2731),       # 8193+ workgroups: the XCD remap is active, tiles end ragged in every slice
    (4, 6, 3, 512, 4, 2049),       # the same with three pipeline stages
    (2, 3, 2, 2048, 8, 1501),      # and for int8 blocks of 2048 with two stages
]


@pytest.mark.parametrize("X,Y,S,block,bits,bps", REORDER_CASES)
def test_qgz_reorder_bit_exact(X, Y, S, block, bits, bps):
    n = X * Y * S * block * bps
    g = workloads.gradients(n, seed=X * 1000 + Y)
    want_codes, want_scales = oracle.qgz_reorder(host_bits(g), oracle.F16, X, Y, S, block, bits)
    cfull, codes = guarded(n * bits // 8, torch.uint8)
    sfull, scales = guarded(n // block, torch.float32)
    zpp.qgz_reorder(g.to(DEV), X, Y, S, block, bits, codes=codes, scales=scales)
    torch.cuda.synchronize()
    assert eq_bytes(scales, want_scales), "scales differ"
    assert eq_bytes(codes, want_codes), "codes differ"
    assert_guards_intact(cfull, n * bits // 8, torch.uint8)
    assert_guards_intact(sfull, n // block, torch.float32)


def test_reorder_index_helpers_match_oracle():
    for X, Y, S in [(2, 2, 1), (8, 48, 1), (3, 5, 4)]:
        for p in range(X * Y * S):
            assert zpp.reorder_source_slice(p, X, Y, S) == oracle.reorder_source_slice(p, X, Y, S)
            assert zpp.reorder_mapped_slice(p, X, Y, S) == oracle.reorder_mapped_slice(p, X, Y, S)
        assert zpp.reorder_source_slice(X * Y * S, X, Y, S) == -1


# ----------------------------------------------------------------------------
# qgZ: the two reduce stages
# ----------------------------------------------------------------------------

def _peer_inputs(K, m, block, bits, seed):
    host, dev = [], []
    for k in range(K):
        g = workloads.gradients(m, seed=seed, tensor_id=k)
        c, s = oracle.qwz_quantize(host_bits(g), oracle.F16, block, bits)
        host.append((c, s))
        dev.append((torch.from_numpy(c).to(DEV), torch.from_numpy(s).to(DEV)))
    return host, dev


INTRA_CASES = [
    # X, block, bits, blocks
    (8, 512, 4, 37),
    (8, 32, 4, 129),
    (2, 64, 4, 65),
    (5, 2048, 4, 3),
    (8, 4096, 4, 3),      # larger than a wave's tile: generic path
    (3, 96, 4, 50),       # not a power of two
    (8, 512, 8, 9),
    (4, 32, 8, 67),
    (7, 2048, 8, 2),
    (1, 256, 4, 11),
    (64, 128, 4, 5),
    (8, 4064, 4, 9),      # one wave per block: 8 rounds, ragged last round
    (5, 2080, 4, 7),
    (8, 2048, 8, 5),      # int8: wider than a wave of 16-byte vectors
    (3, 4096, 8, 3),
    (6, 1056, 8, 13),
    # one wave per block, every number of rounds (1..8) at both widths; peers fetched one
    # ahead in pairs: odd and even counts, one peer, the full table
    (3, 480, 4, 9),
    (4, 992, 4, 7),
    (1, 1536, 4, 5),
    (9, 2016, 4, 6),
    (64, 2528, 4, 3),
    (2, 3072, 4, 4),
    (63, 3552, 4, 2),
    (7, 480, 8, 5),
    (2, 1504, 8, 5),
    (5, 2528, 8, 3),
    (64, 3040, 8, 2),
    (6, 3552, 8, 3),
    (1, 4096, 8, 2),
]


@pytest.mark.parametrize("X,block,bits,blocks", INTRA_CASES)
def test_qgz_intra_reduce_bit_exact(X, block, bits, blocks):
    m = block * blocks
    host, dev = _peer_inputs(X, m, block, bits, seed=X + block)
    want_codes, want_scales = oracle.qgz_intra_reduce([h[0] for h in host], [h[1] for h in host], m, block, bits)
    cfull, codes = guarded(m * bits // 8, torch.uint8)
    sfull, scales = guarded(m // block, torch.float32)
    zpp.qgz_intra_reduce([d[0] for d in dev], [d[1] for d in dev], m, block, bits, codes_out=codes, scales_out=scales)
    torch.cuda.synchronize()
    assert eq_bytes(scales, want_scales), "scales differ"
    assert eq_bytes(codes, want_codes), "codes differ"
    assert_guards_intact(cfull, m * bits // 8, torch.uint8)
    assert_guards_intact(sfull, m // block, torch.float32)


@pytest.mark.parametrize("X,block,blocks,bits", [(8, 4096, 6, 4), (5, 1536, 9, 4), (2, 96, 40, 4), (8, 512, 12, 4),
                                                 (8, 4096, 3, 8), (3, 1504, 5, 8), (8, 512, 12, 8), (4, 128, 40, 8)])
def test_qgz_intra_reduce_with_scales_beyond_the_fused_decode(X, block, blocks, bits):
    """Scales of 2^100 and more (never produced from 16-bit gradients) leave the fused
    decode: the block is then summed by convert and multiply.  One such scale per block, of
    either sign, in some blocks; the outputs are the oracle's bit for bit."""
    m = block * blocks
    host, dev = _peer_inputs(X, m, block, bits, seed=31 + block)
    scales = [h[1].copy() for h in host]
    for b in range(0, blocks, 2):
        scales[(b // 2) % X][b] = np.float32(2.0 ** 101 if b % 4 == 0 else -(2.0 ** 118))
    want_codes, want_scales = oracle.qgz_intra_reduce([h[0] for h in host], scales, m, block, bits)
    got_codes, got_scales = zpp.qgz_intra_reduce([d[0] for d in dev], [torch.from_numpy(s).to(DEV) for s in scales],
                                                 m, block, bits)
    torch.cuda.synchronize()
    assert eq_bytes(got_scales, want_scales), "scales differ"
    assert eq_bytes(got_codes, want_codes), "codes differ"


INTER_CASES = [
    # Y, block, bits, blocks, divisor
    (48, 512, 4, 21, 384.0),
    (2, 32, 4, 131, 1.0),
    (5, 96, 4, 33, 5.0),
    (64, 2048, 4, 2, 512.0),
    (6, 64, 8, 77, 48.0),
    (1, 4096, 8, 3, 3.0),
]


@pytest.mark.parametrize("Y,block,bits,blocks,div", INTER_CASES)
def test_qgz_inter_reduce_bit_exact(Y, block, bits, blocks, div):
    m = block * blocks
    host, dev = _peer_inputs(Y, m, block, bits, seed=Y + block)
    want = oracle.qgz_inter_reduce([h[0] for h in host], [h[1] for h in host], m, block, bits, div)
    ofull, out = guarded(m, torch.float32)
    zpp.qgz_inter_reduce([d[0] for d in dev], [d[1] for d in dev], m, block, bits, div, out=out)
    torch.cuda.synchronize()
    assert eq_bytes(out, want)
    assert_guards_intact(ofull, m, torch.float32)


@pytest.mark.parametrize("X,Y,block", [(2, 2, 32), (8, 6, 512), (4, 3, 64)])
def test_whole_qgz_path_on_simulated_ranks(X, Y, block):
    """W = X*Y ranks as W device buffers; the all-to-alls are pointer offsets.
    Every rank's final partition must equal the oracle's, bit for bit."""
    W, bits = X * Y, 4
    L = block * 3
    n = W * L
    m = n // X
    grads = [workloads.gradients(n, seed=77, tensor_id=r) for r in range(W)]
    # oracle side
    o_first = [oracle.qgz_reorder(host_bits(g), oracle.F16, X, Y, 1, block, bits) for g in grads]
    # GPU side
    d_first = [zpp.qgz_reorder(g.to(DEV), X, Y, 1, block, bits) for g in grads]
    cb, sb = m * bits // 8, m // block
    o_second, d_second = {}, {}
    for node in range(Y):
        for j in range(X):
            o_second[(node, j)] = oracle.qgz_intra_reduce(
                [o_first[node * X + k][0][j * cb:(j + 1) * cb] for k in range(X)],
                [o_first[node * X + k][1][j * sb:(j + 1) * sb] for k in range(X)], m, block, bits)
            d_second[(node, j)] = zpp.qgz_intra_reduce(
                [d_first[node * X + k][0][j * cb:(j + 1) * cb] for k in range(X)],
                [d_first[node * X + k][1][j * sb:(j + 1) * sb] for k in range(X)], m, block, bits)
    cl, sl = L * bits // 8, L // block
    for node in range(Y):
        for j in range(X):
            want = oracle.qgz_inter_reduce(
                [o_second[(i, j)][0][node * cl:(node + 1) * cl] for i in range(Y)],
                [o_second[(i, j)][1][node * sl:(node + 1) * sl] for i in range(Y)], L, block, bits, float(W))
            got = zpp.qgz_inter_reduce(
                [d_second[(i, j)][0][node * cl:(node + 1) * cl] for i in range(Y)],
                [d_second[(i, j)][1][node * sl:(node + 1) * sl] for i in range(Y)], L, block, bits, float(W))
            torch.cuda.synchronize()
            assert eq_bytes(got, want), (node, j)


# ----------------------------------------------------------------------------
# argument handling through the C ABI
# ----------------------------------------------------------------------------

def test_empty_inputs_are_no_ops():
    e16 = torch.empty(0, dtype=torch.float16, device=DEV)
    e8 = torch.empty(0, dtype=torch.uint8, device=DEV)
    e32 = torch.empty(0, dtype=torch.float32, device=DEV)
    zpp.qwz_quantize(e16, 256, 8, codes=e8, scales=e32)
    zpp.qwz_dequantize(e8, e32, 0, 256, 8, out=e16)
    zpp.qgz_reorder(e16, 8, 48, 1, 512, 4, codes=e8, scales=e32)
    one = torch.zeros(16, dtype=torch.uint8, device=DEV)
    onef = torch.zeros(4, dtype=torch.float32, device=DEV)
    zpp.qgz_intra_reduce([one], [onef], 0, 512, 4, codes_out=e8, scales_out=e32)
    zpp.qgz_inter_reduce([one], [onef], 0, 512, 4, 1.0, out=e32)
    torch.cuda.synchronize()


def test_invalid_arguments_return_einval_and_launch_nothing():
    x = torch.zeros(4096, dtype=torch.float16, device=DEV)
    codes = torch.full((4096,), 0xA5, dtype=torch.uint8, device=DEV)
    scales = torch.full((128,), -1.0, dtype=torch.float32, device=DEV)
    bad = [
        lambda: zpp.qwz_quantize(x[:4000], 256, 8, codes=codes, scales=scales),      # n % block
        lambda: zpp.qwz_quantize(x, 48, 8, codes=codes, scales=scales),              # block % 32
        lambda: zpp.qwz_quantize(x, 8192, 8, codes=codes, scales=scales),            # block too large
        lambda: zpp.qwz_quantize(x, 256, 5, codes=codes, scales=scales),             # bits
        lambda: zpp.qwz_quantize(x[1:257], 256, 8, codes=codes, scales=scales),      # misaligned input
        lambda: zpp.qwz_quantize(x, 256, 8, codes=codes[1:], scales=scales),         # misaligned output
        lambda: zpp.qgz_reorder(x, 8, 3, 1, 256, 4, codes=codes, scales=scales),     # n % (X*Y*block)
        lambda: zpp.qgz_reorder(x, 0, 2, 1, 256, 4, codes=codes, scales=scales),
        lambda: zpp.qgz_inter_reduce([codes], [scales], 4096, 256, 4, 0.0),          # divisor
        lambda: zpp.qgz_inter_reduce([codes] * 65, [scales] * 65, 4096, 256, 4, 1.0),  # too many peers
        lambda: zpp.qgz_intra_reduce([], [], 4096, 256, 4),
    ]
    for f in bad:
        with pytest.raises(zpp.ZppError):
            f()
    torch.cuda.synchronize()
    assert bool((codes == 0xA5).all()) and bool((scales == -1.0).all())


def test_results_do_not_depend_on_what_the_output_held_before():
    n, block = 512 * 301, 512
    g = workloads.gradients(n, seed=5).to(DEV)
    a = zpp.qgz_reorder(g, 7, 43, 1, block, 4, codes=torch.zeros(n // 2, dtype=torch.uint8, device=DEV),
                        scales=torch.zeros(n // block, dtype=torch.float32, device=DEV))
    b = zpp.qgz_reorder(g, 7, 43, 1, block, 4, codes=torch.full((n // 2,), 255, dtype=torch.uint8, device=DEV),
                        scales=torch.full((n // block,), float("nan"), dtype=torch.float32, device=DEV))
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))


# ----------------------------------------------------------------------------
# variants by argument
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("W,block,bits", [(8, 64, 4), (48, 512, 4), (16, 128, 8)])
def test_one_hop_all_to_all_reduction(W, block, bits):
    """Sec. 3.3.1: quantize once, all-to-all among all W ranks, dequantize and reduce in
    full precision.  No reordering is needed; the reduce is qgz_inter_reduce with W peers."""
    L = block * 5
    n = W * L
    grads = [workloads.gradients(n, seed=55, tensor_id=r) for r in range(W)]
    o_q = [oracle.qwz_quantize(host_bits(g), oracle.F16, block, bits) for g in grads]
    d_q = [zpp.qwz_quantize(g.to(DEV), block, bits) for g in grads]
    cl, sl = L * bits // 8, L // block
    exact = np.mean(np.stack([g.double().numpy() for g in grads]), axis=0)
    for r in (0, W // 2, W - 1):
        want = oracle.qgz_inter_reduce([c[r * cl:(r + 1) * cl] for c, _ in o_q], [s[r * sl:(r + 1) * sl] for _, s in o_q],
                                       L, block, bits, float(W))
        got = zpp.qgz_inter_reduce([c[r * cl:(r + 1) * cl] for c, _ in d_q], [s[r * sl:(r + 1) * sl] for _, s in d_q],
                                   L, block, bits, float(W))
        torch.cuda.synchronize()
        assert eq_bytes(got, want)
        # and it is the mean of the ranks' slices up to the quantization step
        step = np.mean(np.stack([np.repeat(s[r * sl:(r + 1) * sl], block) for _, s in o_q]), axis=0) / 2
        assert np.all(np.abs(want - exact[r * L:(r + 1) * L]) <= step * (1 + 1e-3) + 1e-12)


@pytest.mark.parametrize("dtype", [oracle.BF16, oracle.F32])
def test_qgz_reorder_accepts_other_gradient_dtypes(dtype):
    X, Y, block, bits = 4, 6, 256, 8
    n = X * Y * block * 7
    g = workloads.gradients(n, seed=56, dtype=TORCH_DT[dtype])
    want_codes, want_scales = oracle.qgz_reorder(host_bits(g), dtype, X, Y, 1, block, bits)
    codes, scales = zpp.qgz_reorder(g.to(DEV), X, Y, 1, block, bits)
    torch.cuda.synchronize()
    assert eq_bytes(codes, want_codes) and eq_bytes(scales, want_scales)


def test_reduce_stages_with_very_large_scales():
    """Scales of 2^100 and above take the plain decode branch of the reduce kernels."""
    block, m, K = 512, 512 * 9, 5
    host, dev = [], []
    rng = np.random.default_rng(4)
    for k in range(K):
        x = (rng.standard_normal(m) * 2.0 ** (96 + 6 * k)).astype(np.float32)      # block maxima up to ~2^124
        c, s = oracle.qwz_quantize(x, oracle.F32, block, 4)
        host.append((c, s))
        dev.append((torch.from_numpy(c).to(DEV), torch.from_numpy(s).to(DEV)))
    assert max(float(s.max()) for _, s in host) > 2.0 ** 110
    wc, ws = oracle.qgz_intra_reduce([c for c, _ in host], [s for _, s in host], m, block, 4)
    gc, gs = zpp.qgz_intra_reduce([c for c, _ in dev], [s for _, s in dev], m, block, 4)
    wo = oracle.qgz_inter_reduce([c for c, _ in host], [s for _, s in host], m, block, 4, 4.0)
    go = zpp.qgz_inter_reduce([c for c, _ in dev], [s for _, s in dev], m, block, 4, 4.0)
    torch.cuda.synchronize()
    assert eq_bytes(gc, wc) and eq_bytes(gs, ws) and eq_bytes(go, wo)


@pytest.mark.parametrize("bits", [8, 4])
def test_block_quotient_sequences_equal_division_for_every_mantissa(bits):
    """The encoders' short fma sequences for absmax/qmax and qmax/absmax against plain
    division: all 2^23 mantissas at the ends of the range they are used in, at 1.0,
    at typical weight and gradient magnitudes, and at the binades next to qmax."""
    for exponent in (-100, -99, -24, -14, -10, -6, -1, 0, 1, 2, 3, 6, 7, 15, 64, 98, 99):
        assert diagnostics.selfcheck_block_scale(bits, exponent) == (0, 0), exponent


@pytest.mark.parametrize("bits,block", [(4, 512), (4, 96), (8, 2048), (8, 160)])
def test_decoders_accept_every_code_value(bits, block):
    """Codes that no quantizer writes (nibble 0x8 = -8, byte 0x80 = -128) are still two's
    complement to the decode and to both reduce stages: random bytes as codes."""
    rng = np.random.default_rng(4242 + bits + block)
    K, blocks = 5, 37
    n = block * blocks
    codes = [rng.integers(0, 256, size=n * bits // 8, dtype=np.uint8) for _ in range(K)]
    for c in codes:
        c[:16] = 0x88 if bits == 4 else 0x80                 # a run of the most negative code
    scales = [(10.0 ** rng.uniform(-9, 4, size=blocks)).astype(np.float32) for _ in range(K)]   # fp16 decodes span zero, subnormals and overflow
    dcodes = [torch.from_numpy(c).to(DEV) for c in codes]
    dscales = [torch.from_numpy(s).to(DEV) for s in scales]
    for odt in (oracle.F32, oracle.F16, oracle.BF16):
        y = torch.empty(n, dtype=TORCH_DT[odt], device=DEV)
        zpp.qwz_dequantize(dcodes[0], dscales[0], n, block, bits, out=y)
        torch.cuda.synchronize()
        assert eq_bytes(y, oracle.qwz_dequantize(codes[0], scales[0], n, block, bits, odt))
    hc, hs = oracle.qgz_intra_reduce(codes, scales, n, block, bits)
    dc, ds = zpp.qgz_intra_reduce(dcodes, dscales, n, block, bits)
    torch.cuda.synchronize()
    assert eq_bytes(ds, hs) and eq_bytes(dc, hc)
    out = zpp.qgz_inter_reduce(dcodes, dscales, n, block, bits, 3.0)
    torch.cuda.synchronize()
    assert eq_bytes(out, oracle.qgz_inter_reduce(codes, scales, n, block, bits, 3.0))


@pytest.mark.parametrize("block", [512, 96, 4096, 64, 256])
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("K", [1, 3])
def test_reduce_stages_return_plus_zero_for_zero_products(bits, K, block):
    """Products that are -0 (code 0 times a negative scale, a negative code times a zero scale
    of either sign) must not leak their sign: every sum starts from +0, so both stages return
    +0 bits, exactly as the oracle does, also with a single peer, in every kernel the block
    size selects, and also where a scale of 2^101 sends a block to the convert-and-multiply path."""
    blocks = 8
    n = block * blocks
    rng = np.random.default_rng(99 + bits + K)
    codes, scales = [], []
    for k in range(K):
        c = np.zeros(n * bits // 8, dtype=np.uint8)
        s = np.zeros(blocks, dtype=np.float32)
        s[0] = -0.25                     # block 0: code 0, negative scale
        s[1] = 0.0                       # block 1: negative codes, +0 scale
        s[2] = -0.0                      # block 2: negative codes, -0 scale
        s[3] = -0.0                      # block 3: positive codes, -0 scale
        s[4] = 0.5                       # block 4: ordinary values
        s[5] = -1e-3                     # block 5: ordinary values, negative scale
        s[6] = -(2.0 ** 101)             # block 6: code 0, a negative scale beyond the fused decode
        s[7] = 2.0 ** 101                # block 7: ordinary values at such a scale
        per = block * bits // 8
        c[per:3 * per] = 0x99 if bits == 4 else 0xF9           # -7 in every field
        c[3 * per:4 * per] = 0x33 if bits == 4 else 0x05
        c[4 * per:6 * per] = rng.integers(0, 256, size=2 * per, dtype=np.uint8)
        c[7 * per:] = rng.integers(0, 256, size=per, dtype=np.uint8)
        codes.append(c)
        scales.append(s)
    dcodes = [torch.from_numpy(c).to(DEV) for c in codes]
    dscales = [torch.from_numpy(s).to(DEV) for s in scales]
    want = oracle.qgz_inter_reduce(codes, scales, n, block, bits, 1.0)
    assert not np.signbit(want[:4 * block]).any() and (want[:4 * block] == 0).all()
    assert not np.signbit(want[6 * block:7 * block]).any() and (want[6 * block:7 * block] == 0).all()
    got = zpp.qgz_inter_reduce(dcodes, dscales, n, block, bits, 1.0)
    torch.cuda.synchronize()
    assert eq_bytes(got, want)
    want5 = oracle.qgz_inter_reduce(codes, scales, n, block, bits, 5.0)
    got5 = zpp.qgz_inter_reduce(dcodes, dscales, n, block, bits, 5.0)
    torch.cuda.synchronize()
    assert eq_bytes(got5, want5)
    hc, hs = oracle.qgz_intra_reduce(codes, scales, n, block, bits)
    dc, ds = zpp.qgz_intra_reduce(dcodes, dscales, n, block, bits)
    torch.cuda.synchronize()
    assert eq_bytes(ds, hs) and eq_bytes(dc, hc)


@pytest.mark.parametrize("divisor", [384.0, 3.0, 48.0, 5.0, 7.0, 1000.0, 0.3, 65535.0, 1.0 / 1024 + 1e-6])
def test_short_division_equals_division_for_every_dividend(divisor):
    """The inter-node stage's division by a launch constant (reciprocal prepared on the host,
    two exact-remainder corrections) against the fp32 division, for every dividend in the range
    the kernel uses it on."""
    assert diagnostics.selfcheck_divide(divisor) == 0


@pytest.mark.parametrize("Y,blocks,div", [(48, 1152, 384.0), (5, 8192, 5.0), (4, 8193, 384.0), (3, 9215, 3.0),
                                          (6, 9216, 384.0), (3, 10239, 7.0), (3, 10240, 3.0), (3, 10241, 7.0), (4, 12288, 4.0), (3, 12289, 0.37),
                                          (17, 1537, 17.0), (64, 1031, 1e-5), (1, 9216, 384.0), (2, 9216, 3.0), (64, 9216, 64.0),
                                          (1, 10240, 5.0)])
def test_qgz_inter_reduce_across_launch_shapes(Y, blocks, div):
    """Sizes on both sides of the limits at which the launch changes the number of vectors a
    wave takes: one up to 8192 wave tiles and above 12288, two or three in between (9216 tiles
    is the benchmark step's launch); odd counts end inside a wave's tile.  The divisors take the
    short division, the reciprocal multiply (powers of two) and the plain division (1e-5)."""
    block, bits = 512, 4
    m = block * blocks
    host, dev = _peer_inputs(Y, m, block, bits, seed=Y + blocks)
    want = oracle.qgz_inter_reduce([h[0] for h in host], [h[1] for h in host], m, block, bits, div)
    ofull, out = guarded(m, torch.float32)
    zpp.qgz_inter_reduce([d[0] for d in dev], [d[1] for d in dev], m, block, bits, div, out=out)
    torch.cuda.synchronize()
    assert eq_bytes(out, want)
    assert_guards_intact(ofull, m, torch.float32)


@pytest.mark.parametrize("Y,block,bits,blocks,div", [
    (48, 1536, 4, 7, 384.0),       # 12 rows of 128 elements per block
    (5, 384, 4, 33, 5.0),
    (64, 3200, 4, 3, 3.0),
    (3, 1536, 4, 3072, 384.0),     # 9216 wave tiles: three vectors per wave
    (2, 640, 4, 8192, 7.0),        # 10240 wave tiles: two vectors per wave
    (2, 1536, 4, 4097, 3.0),       # 12291 wave tiles: one vector per wave, large grid
    (6, 192, 8, 50, 48.0),         # int8: rows of 64 elements
    (3, 4032, 8, 2, 7.25),
    (2, 576, 8, 4096, 24.0),       # int8, 9216 wave tiles
])
def test_qgz_inter_reduce_blocks_of_whole_rows_that_are_not_powers_of_two(Y, block, bits, blocks, div):
    """Blocks that are a whole number of 16-lane rows (128 int4 or 64 int8 elements) but not a
    power of two take the same kernels as the powers of two, with the block of a row found by
    a division prepared on the host; every launch shape of those kernels."""
    m = block * blocks
    host, dev = _peer_inputs(Y, m, block, bits, seed=Y + block)
    want = oracle.qgz_inter_reduce([h[0] for h in host], [h[1] for h in host], m, block, bits, div)
    ofull, out = guarded(m, torch.float32)
    zpp.qgz_inter_reduce([d[0] for d in dev], [d[1] for d in dev], m, block, bits, div, out=out)
    torch.cuda.synchronize()
    assert eq_bytes(out, want)
    assert_guards_intact(ofull, m, torch.float32)


@pytest.mark.parametrize("block,elements", [
    (256, 512 * 9216), (256, 512 * 10240), (256, 512 * 12289), (256, 512 * 8192 + 256),   # vectors of two code dwords
    (384, 512 * 9216), (1152, 1152 * 4551),                                               # the same, block not a power of two
    (64, 256 * 9216), (64, 256 * 10240), (64, 256 * 12289),                               # vectors of one code dword
    (192, 256 * 9216), (320, 320 * 8193),
])
def test_qgz_inter_reduce_int8_across_launch_shapes(block, elements):
    """The same launch shapes for int8 codes.  Blocks that are multiples of 128 take vectors of
    two code dwords (a wave tile is 512 elements), other multiples of 64 vectors of one (256
    elements); one, two and three vectors per wave in each form."""
    bits, Y = 8, 3
    m = elements
    assert m % block == 0
    host, dev = _peer_inputs(Y, m, block, bits, seed=block)
    want = oracle.qgz_inter_reduce([h[0] for h in host], [h[1] for h in host], m, block, bits, 24.0)
    ofull, out = guarded(m, torch.float32)
    zpp.qgz_inter_reduce([d[0] for d in dev], [d[1] for d in dev], m, block, bits, 24.0, out=out)
    torch.cuda.synchronize()
    assert eq_bytes(out, want)
    assert_guards_intact(ofull, m, torch.float32)


@pytest.mark.parametrize("blocks,huge,bits", [(40, 2.0 ** 70, 4), (9216, 2.0 ** 70, 4), (9216, 2.0 ** 101, 4), (10240, 2.0 ** 120, 4),
                                              (40, 2.0 ** 101, 8), (9216, 2.0 ** 70, 8), (9216, 2.0 ** 110, 8), (10240, 2.0 ** 101, 8)])
def test_qgz_inter_reduce_with_scales_outside_the_short_division_range(blocks, huge, bits):
    """Tiny (2^-40) and subnormal scales, and huge ones, keep the plain division; scales of
    2^100 and more also leave the fused decode (every lane then decodes with its own scale
    loads, by convert and multiply), at one and at several vectors per wave, for both code
    widths (every code value occurs, -8 and -128 included).  The result is the oracle's bit for bit."""
    block, Y = (512 if bits == 4 else 256), 6
    m = block * blocks
    rng = np.random.default_rng(7)
    codes = [rng.integers(0, 256, size=m * bits // 8, dtype=np.uint8) for _ in range(Y)]
    scales = []
    for k in range(Y):
        s = (10.0 ** rng.uniform(-4, 0, size=blocks)).astype(np.float32)
        s[3 * k % blocks] = np.float32(2.0 ** -40)
        s[(3 * k + 1) % blocks] = np.float32(1e-41)          # subnormal
        s[(3 * k + 2) % blocks] = np.float32(huge)
        s[(977 * k + 5) % blocks] = np.float32(-huge)
        scales.append(s)
    want = oracle.qgz_inter_reduce(codes, scales, m, block, bits, 384.0)
    got = zpp.qgz_inter_reduce([torch.from_numpy(c).to(DEV) for c in codes], [torch.from_numpy(s).to(DEV) for s in scales],
                               m, block, bits, 384.0)
    torch.cuda.synchronize()
    assert eq_bytes(got, want)
