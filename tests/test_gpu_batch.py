"""GPU parity, batch cost models: the HIP kernels behind cc_ring_cost_batch / cc_rd_cost_batch /
cc_init_tours / cc_validate_matrix against the CPU oracle, element by element (integers: bit-exact)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2105_14088_amd as cc
from gen import COST_MAX, WORKLOADS, make_matrix, random_matrix, random_perms
from gpu_util import dev, gpu_rd, gpu_ring, report, say

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]


def test_workload1_all_2520_rings_and_4096_seeded_orders():
    say("C1: N=8, 2520 rings + 4096 seeded orders, ring sum")
    c = make_matrix(1)
    ex = oracle.exhaustive_rings(c, oracle.SUM, half_only=True, keep_all=True)
    got = gpu_ring(c, ex["rings"], cc.CC_RING_SUM)
    assert np.array_equal(got, ex["costs"])
    k = int(np.argmin(got))                      # first minimum = first minimiser in enumeration order
    assert got[k] == ex["best_cost"] and np.array_equal(ex["rings"][k], ex["best_ring"])
    seed = WORKLOADS[1].search_seed
    tours = cc.cc_init_tours(8, 4096, seed)
    torch.cuda.synchronize()
    tours = tours.cpu().numpy()
    assert np.array_equal(tours, oracle.init_tours(seed, 8, 4096))
    assert np.array_equal(gpu_ring(c, tours, cc.CC_RING_SUM), oracle.ring_cost_batch(c, tours, oracle.SUM))
    assert np.array_equal(gpu_ring(c, tours, cc.CC_RING_MAX), oracle.ring_cost_batch(c, tours, oracle.MAX))


@pytest.mark.parametrize("n", [2, 3, 5, 8, 13, 16, 32, 64, 100, 128, 256, 1000, 1024])
@pytest.mark.parametrize("obj", [0, 1])
def test_ring_batch_sizes_and_ragged_tails(n, obj):
    # batch sizes that leave partial wave-loads, partial unrolled groups and a single order
    c = random_matrix(n, 300 + n, symmetric=False, lo=0, hi=COST_MAX if n in (13, 64) else 6000)
    for b in (1, 3, 67, 1029):
        say(f"ring batch N={n} obj={obj} B={b}")
        perms = random_perms(n, b, seed=n + b)
        assert np.array_equal(gpu_ring(c, perms, obj), oracle.ring_cost_batch(c, perms, obj))


@pytest.mark.parametrize("n", [2, 3, 13, 16, 32, 64, 100, 128, 200, 256])
@pytest.mark.parametrize("obj", [0, 1])
def test_ring_batch_u8_orders(n, obj):
    c = random_matrix(n, 700 + n, symmetric=False, lo=0, hi=COST_MAX if n in (13, 64) else 6000)
    for b in (1, 3, 67, 1029, 4100):
        say(f"ring batch, one byte per rank, N={n} obj={obj} B={b}")
        perms = random_perms(n, b, seed=n + b)
        out = cc.cc_ring_cost_batch_u8(dev(c), dev(perms.astype(np.uint8)), obj)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), oracle.ring_cost_batch(c, perms, obj))


def test_ring_batch_u8_unaligned_out_of_range_and_full_size():
    say("ring batch u8: unaligned stream, out-of-range bytes, 2^20 orders")
    c = make_matrix(2)
    perms = random_perms(64, 33, seed=2)
    flat = torch.empty(33 * 64 + 1, dtype=torch.uint8, device="cuda")
    view = flat[1:].view(33, 64)
    view.copy_(dev(perms.astype(np.uint8)))
    out = cc.cc_ring_cost_batch_u8(dev(c), view, 0)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), oracle.ring_cost_batch(c, perms, 0))
    bad = perms.astype(np.uint8)
    bad[::2, 5] = 255                                   # not a rank: result unspecified, access must stay in bounds
    cc.cc_ring_cost_batch_u8(dev(c), dev(bad), 1)
    torch.cuda.synchronize()
    B = 1 << 20
    tours = cc.cc_init_tours(64, B, WORKLOADS[2].search_seed)
    want = cc.cc_ring_cost_batch(dev(c), tours, 0)
    got = cc.cc_ring_cost_batch_u8(dev(c), tours.to(torch.uint8), 0)
    torch.cuda.synchronize()
    assert torch.equal(want, got)
    rows = np.arange(0, B, 4099)
    assert np.array_equal(got.cpu().numpy()[rows], oracle.ring_cost_batch(c, tours.cpu().numpy()[rows], 0))


@pytest.mark.parametrize("n", [2, 13, 64, 257, 300, 512, 1024])
@pytest.mark.parametrize("obj", [0, 1])
def test_ring_batch_u16_orders(n, obj):
    """Two bytes per rank: any N; also an odd element offset of the stream and ranks out of range (access must stay
    in bounds)."""
    c = random_matrix(n, 1700 + n, symmetric=False, lo=0, hi=COST_MAX if n in (13, 64) else 6000)
    for b in (1, 3, 67, 1029):
        say(f"ring batch, two bytes per rank, N={n} obj={obj} B={b}")
        perms = random_perms(n, b, seed=n + b)
        out = cc.cc_ring_cost_batch_u16(dev(c), dev(perms.astype(np.int16)), obj)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), oracle.ring_cost_batch(c, perms, obj))
    perms = random_perms(n, 9, seed=n)
    flat = torch.empty(9 * n + 1, dtype=torch.int16, device="cuda")
    view = flat[1:].view(9, n)
    view.copy_(dev(perms.astype(np.int16)))
    out = cc.cc_ring_cost_batch_u16(dev(c), view, obj)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), oracle.ring_cost_batch(c, perms, obj))
    bad = perms.astype(np.int16)
    bad[::2, 1] = -1                                    # 65535 as a rank: result unspecified
    cc.cc_ring_cost_batch_u16(dev(c), dev(bad), obj)
    torch.cuda.synchronize()


@pytest.mark.parametrize("obj", [0, 1])
def test_ring_batch_n256_large_batches_lds_kernel_and_its_fallback(obj):
    """N = 256 from 32768 orders on: the matrix as 16-bit entries in LDS; a matrix with an entry of 2^16 is scored
    through L2 by the same kernel.  A batch size that is no multiple of the kernel's step, every order compared."""
    B = 32768 + 4099
    perms = random_perms(256, B, seed=77 + obj)
    for top, symmetric in (((1 << 16) - 1, False), (1 << 16, False), (2000, True)):
        say(f"ring batch N=256 B={B} obj={obj} largest entry {top}")
        c = random_matrix(256, 4000 + top % 13, symmetric=symmetric, lo=max(0, top - 40000), hi=top)
        c[7, 9] = top
        if symmetric:
            c[9, 7] = top
        assert np.array_equal(gpu_ring(c, perms, obj), oracle.ring_cost_batch(c, perms, obj))


@pytest.mark.parametrize("n,base", [(128, 2), (256, 2), (256, 4)])
def test_large_batches_n128_n256_matrix_in_lds_and_its_fallback(n, base):
    """Halving-doubling (base 2) and BCube base 4 from 32768 orders on: folded 16-bit matrix in LDS; with an entry of
    2^16 the same kernel scores through L2.  With and without round weights, every order compared."""
    B = 32768 + 1031
    perms = random_perms(n, B, seed=5 * n + base)
    rounds = 0
    while base ** rounds < n:
        rounds += 1
    weights = np.random.default_rng(n + base).integers(0, 1 << 20, size=rounds).astype(np.int32)
    perms_dev, w_dev = dev(perms), dev(weights)
    for top, symmetric in (((1 << 16) - 1, False), (1 << 16, False), (900, True)):
        say(f"large batch N={n} base={base} B={B} largest entry {top}")
        c = random_matrix(n, 6000 + n + top % 17, symmetric=symmetric, lo=max(0, top - 50000), hi=top)
        c[2, 5] = top
        if symmetric:
            c[5, 2] = top
        c_dev = dev(c)
        plain = cc.cc_bcube_cost_batch(c_dev, base, perms_dev)
        weighted = cc.cc_bcube_cost_batch_weighted(c_dev, base, w_dev, perms_dev)
        torch.cuda.synchronize()
        assert np.array_equal(plain.cpu().numpy(), oracle.bcube_cost_batch(c, base, perms))
        assert np.array_equal(weighted.cpu().numpy(), oracle.bcube_cost_weighted_batch(c, base, weights, perms))
        if base == 2:
            rd = cc.cc_rd_cost_batch(c_dev, perms_dev)
            torch.cuda.synchronize()
            assert np.array_equal(rd.cpu().numpy(), oracle.rd_cost_batch(c, perms))


def test_ring_batch_empty_and_unaligned():
    c = random_matrix(64, 1, symmetric=True)
    say("ring batch B=0")
    out = cc.cc_ring_cost_batch(dev(c), torch.empty((0, 64), dtype=torch.int32, device="cuda"), 0)
    torch.cuda.synchronize()
    assert out.numel() == 0
    say("ring batch, order stream not 16-byte aligned")
    perms = random_perms(64, 33, seed=2)
    flat = torch.empty(33 * 64 + 1, dtype=torch.int32, device="cuda")
    view = flat[1:].view(33, 64)
    view.copy_(dev(perms))
    out = cc.cc_ring_cost_batch(dev(c), view, 0)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), oracle.ring_cost_batch(c, perms, 0))


@pytest.mark.parametrize("wid", [2, 3])
@pytest.mark.parametrize("obj", [0, 1])
def test_headline_batch_2pow20_orders_n64_full(wid, obj):
    """The batch-evaluation headline case at full size: 2^20 seeded orders at N=64, matrices 2 and 3, sum and
    max-hop; the oracle generates all 2^20 orders and scores every one of them."""
    say(f"M64: N=64 matrix {wid} obj={obj} B=2^20, every order and cost compared")
    c = make_matrix(wid)
    B = 1 << 20
    seed = WORKLOADS[wid].search_seed
    tours = cc.cc_init_tours(64, B, seed)
    out = cc.cc_ring_cost_batch(dev(c), tours, obj)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    th = tours.cpu().numpy()
    want_orders = oracle.init_tours(seed, 64, B)
    assert np.array_equal(th, want_orders)
    assert np.array_equal(got, oracle.ring_cost_batch(c, want_orders, obj))
    report(f"M64 (matrix {wid}, objective {obj}): {B} of {B} orders and costs compared")


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64, 128, 256, 512, 1024])
def test_rd_batch(n):
    c = random_matrix(n, 500 + n, symmetric=False, lo=0, hi=COST_MAX if n == 64 else 9000)
    for b in (1, 5, 259):
        say(f"rd batch N={n} B={b}")
        perms = random_perms(n, b, seed=n * 3 + b)
        assert np.array_equal(gpu_rd(c, perms), oracle.rd_cost_batch(c, perms))


@pytest.mark.parametrize("n", [128, 256, 512, 1024])
def test_rd_batch_with_workspace_folded_copy_and_its_fallback(n):
    """cc_rd_cost_batch_ex: symmetric and asymmetric matrices, the largest entry one below 2^16 (folded 16-bit copy, one
    look-up per link) and at 2^16 (the look-up per rank of cc_rd_cost_batch), a caller's workspace used twice, and
    the plain call on the same inputs."""
    ws = torch.empty(cc.cc_rd_batch_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    for top, symmetric in (((1 << 16) - 1, False), ((1 << 16) - 1, True), (1 << 16, False), (40, True)):
        say(f"rd batch with workspace N={n} largest entry {top} symmetric={symmetric}")
        c = random_matrix(n, 600 + n + top % 7, symmetric=symmetric, lo=max(0, top - 30000), hi=top)
        c[1, 2] = top
        if symmetric:
            c[2, 1] = top
        perms = random_perms(n, 131, seed=n + top % 11)
        want = oracle.rd_cost_batch(c, perms)
        c_dev, perms_dev = dev(c), dev(perms)
        got = cc.cc_rd_cost_batch(c_dev, perms_dev, workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), want)
        plain = torch.empty(131, dtype=torch.int64, device="cuda")
        rc = cc.lib().cc_rd_cost_batch(c_dev.data_ptr(), n, perms_dev.data_ptr(), 131, plain.data_ptr(),
                                       torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert rc == 0 and np.array_equal(plain.cpu().numpy(), want)


@pytest.mark.parametrize("n,base", [(4, 4), (16, 4), (64, 4), (256, 4), (1024, 4), (9, 3), (27, 3), (243, 3), (729, 3),
                                    (64, 8), (512, 8), (25, 5), (625, 5), (32, 32), (1024, 32), (64, 2), (7, 7)])
def test_bcube_batch(n, base):
    c = random_matrix(n, 900 + n, symmetric=False, lo=0, hi=COST_MAX if n == 64 else 9000)
    for b in (1, 5, 259) + ((20011,) if n == 64 else ()):      # N = 64: enough orders for several per wave
        say(f"bcube batch N={n} base={base} B={b}")
        perms = random_perms(n, b, seed=n * 5 + b)
        out = cc.cc_bcube_cost_batch(dev(c), base, dev(perms))
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), oracle.bcube_cost_batch(c, base, perms))


@pytest.mark.parametrize("n,base", [(64, 2), (1024, 2), (128, 2), (64, 4), (256, 4), (243, 3), (8, 8)])
def test_bcube_weighted_batch(n, base):
    c = random_matrix(n, 1500 + n, symmetric=False, lo=0, hi=COST_MAX if n == 64 else 9000)
    rounds = 0
    while base ** rounds < n:
        rounds += 1
    rng = np.random.default_rng(n + base)
    for weights in (np.ones(rounds, dtype=np.int32), rng.integers(0, 1 << 20, size=rounds).astype(np.int32),
                    np.array([(1 << 30) >> k for k in range(rounds)], dtype=np.int32)):
        say(f"bcube weighted N={n} base={base} weights={weights.tolist()}")
        perms = random_perms(n, 131, seed=n + rounds)
        out = cc.cc_bcube_cost_batch_weighted(dev(c), base, dev(weights), dev(perms))
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), oracle.bcube_cost_weighted_batch(c, base, weights, perms))


def test_n64_cost_models_on_an_order_stream_that_is_not_16_byte_aligned():
    """N = 64: the one-order-per-lane kernels need 16-byte aligned orders; a stream that starts one element later
    takes the one-order-per-wave kernels.  Both against the oracle, on a batch with a ragged last group of 64."""
    say("N=64 halving-doubling / BCube base 4 / double binary tree: aligned and unaligned order streams, B = 1000")
    c = random_matrix(64, 321, symmetric=False, lo=0, hi=COST_MAX)
    perms = random_perms(64, 1000, seed=12)
    flat = torch.zeros(1 + perms.size, dtype=torch.int32, device="cuda")
    flat[1:] = torch.from_numpy(perms.reshape(-1)).cuda()
    shifted = flat[1:].view(1000, 64)
    assert shifted.data_ptr() % 16 == 4
    c_dev, aligned = dev(c), dev(perms)
    for view in (aligned, shifted):
        rd = torch.empty(1000, dtype=torch.int64, device="cuda")
        bc = torch.empty(1000, dtype=torch.int64, device="cuda")
        tr = torch.empty(1000, dtype=torch.int64, device="cuda")
        L, st = cc.lib(), torch.cuda.current_stream().cuda_stream
        assert L.cc_rd_cost_batch(c_dev.data_ptr(), 64, view.data_ptr(), 1000, rd.data_ptr(), st) == 0
        assert L.cc_bcube_cost_batch(c_dev.data_ptr(), 64, 4, view.data_ptr(), 1000, bc.data_ptr(), st) == 0
        assert L.cc_dbt_cost_batch(c_dev.data_ptr(), 64, view.data_ptr(), 1000, tr.data_ptr(), st) == 0
        torch.cuda.synchronize()
        assert np.array_equal(rd.cpu().numpy(), oracle.rd_cost_batch(c, perms))
        assert np.array_equal(bc.cpu().numpy(), oracle.bcube_cost_batch(c, 4, perms))
        assert np.array_equal(tr.cpu().numpy(), oracle.dbt_cost_batch(c, perms))


@pytest.mark.parametrize("n,base", [(256, 4), (1024, 4), (128, 2), (512, 2), (243, 3), (16, 4)])
def test_bcube_with_workspace_folded_copy_and_its_fallback(n, base):
    """cc_bcube_cost_batch_ex with and without round weights: the largest entry one below 2^16 (folded copy where
    the size has one) and at 2^16 (per-rank kernel), symmetric and not; and the call without workspace on the same
    inputs."""
    rounds = 0
    while base ** rounds < n:
        rounds += 1
    weights = np.random.default_rng(n).integers(0, 1 << 20, size=rounds).astype(np.int32)
    ws = torch.empty(cc.cc_rd_batch_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    for top, symmetric in (((1 << 16) - 1, False), ((1 << 16) - 1, True), (1 << 16, False), (3, False)):
        say(f"bcube with workspace N={n} base={base} largest entry {top} symmetric={symmetric}")
        c = random_matrix(n, 700 + n + top % 7, symmetric=symmetric, lo=max(0, top - 30000), hi=top)
        c[0, 1] = top
        if symmetric:
            c[1, 0] = top
        perms = random_perms(n, 131, seed=n + top % 13)
        c_dev, perms_dev, w_dev = dev(c), dev(perms), dev(weights)
        got = cc.cc_bcube_cost_batch(c_dev, base, perms_dev, workspace=ws)
        got_w = cc.cc_bcube_cost_batch_weighted(c_dev, base, w_dev, perms_dev, workspace=ws)
        plain = torch.empty(131, dtype=torch.int64, device="cuda")
        rc = cc.lib().cc_bcube_cost_batch(c_dev.data_ptr(), n, base, perms_dev.data_ptr(), 131, plain.data_ptr(),
                                          torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        want = oracle.bcube_cost_batch(c, base, perms)
        assert np.array_equal(got.cpu().numpy(), want)
        assert np.array_equal(got_w.cpu().numpy(), oracle.bcube_cost_weighted_batch(c, base, weights, perms))
        assert rc == 0 and np.array_equal(plain.cpu().numpy(), want)


def test_bcube_base4_n1024_16384_orders():
    """Full-size case: B = 4 (the paper's BCube base) on 16384 seeded orders at N = 1024, sampled against the oracle."""
    say("bcube batch N=1024 base=4 B=16384")
    c = make_matrix(5)
    seed = WORKLOADS[5].search_seed
    B = 16384
    tours = cc.cc_init_tours(1024, B, seed)
    out = cc.cc_bcube_cost_batch(dev(c), 4, tours)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    rows = np.unique(np.concatenate([np.arange(0, B, 67), np.arange(B - 8, B)]))
    th = tours[torch.from_numpy(rows).cuda()].cpu().numpy()
    assert np.array_equal(got[rows], oracle.bcube_cost_batch(c, 4, th))


@pytest.mark.parametrize("n", [2, 3, 4, 5, 7, 8, 13, 63, 64, 65, 100, 128, 255, 256, 1000, 1023, 1024])
def test_dbt_batch(n):
    c = random_matrix(n, 1200 + n, symmetric=False, lo=0, hi=COST_MAX if n in (64, 1024) else 9000)
    for b in (1, 5, 259):
        say(f"dbt batch N={n} B={b}")
        perms = random_perms(n, b, seed=n * 7 + b)
        out = cc.cc_dbt_cost_batch(dev(c), dev(perms))
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), oracle.dbt_cost_batch(c, perms))


def test_dbt_n64_2_20_orders():
    """Full size: 2^20 seeded orders at N = 64 (matrix of workload 2), sampled against the oracle."""
    say("dbt batch N=64 B=2^20")
    c = make_matrix(2)
    seed = WORKLOADS[2].search_seed
    B = 1 << 20
    tours = cc.cc_init_tours(64, B, seed)
    out = cc.cc_dbt_cost_batch(dev(c), tours)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    rows = np.unique(np.concatenate([np.arange(0, B, 1021), np.arange(B - 8, B)]))
    th = tours[torch.from_numpy(rows).cuda()].cpu().numpy()
    assert np.array_equal(got[rows], oracle.dbt_cost_batch(c, th))


def test_workload5_rd_65536_orders_n1024_full():
    """Full size: 65536 seeded orders at N=1024; the oracle generates and scores all of them.  Both forms of the
    call (with the folded-matrix workspace, as the Python wrapper issues it, and cc_rd_cost_batch without)."""
    say("C5: rd batch N=1024 B=65536, every order and cost compared")
    c = make_matrix(5)
    seed = WORKLOADS[5].search_seed
    B = 65536
    tours = cc.cc_init_tours(1024, B, seed)
    cd = dev(c)
    out = cc.cc_rd_cost_batch(cd, tours)
    plain = torch.empty(B, dtype=torch.int64, device="cuda")
    rc = cc.lib().cc_rd_cost_batch(ctypes.c_void_p(cd.data_ptr()), 1024, ctypes.c_void_p(tours.data_ptr()), B,
                                   ctypes.c_void_p(plain.data_ptr()),
                                   ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0
    torch.cuda.synchronize()
    want_orders = oracle.init_tours(seed, 1024, B)
    assert np.array_equal(tours.cpu().numpy(), want_orders)
    want = oracle.rd_cost_batch(c, want_orders)
    assert np.array_equal(out.cpu().numpy(), want)
    assert np.array_equal(plain.cpu().numpy(), want)
    report(f"C5 (N=1024 halving-doubling batch): {B} of {B} orders and costs compared, both call forms")


@pytest.mark.parametrize("n", [2, 3, 8, 13, 64, 65, 256, 1024])
def test_init_tours_match_oracle(n):
    say(f"init tours N={n}")
    for first, count in ((0, 1), (0, 300), (4093, 10), ((1 << 32) - 5, 5)):
        t = cc.cc_init_tours(n, count, 0xC0FFEE02, first=first)
        torch.cuda.synchronize()
        assert np.array_equal(t.cpu().numpy(), oracle.init_tours(0xC0FFEE02, n, count, first=first))


def test_out_of_range_indices_stay_memory_safe():
    """Orders with indices outside [0, N) give unspecified costs but must not fault."""
    for n in (13, 64, 256):
        say(f"ring/rd batch with out-of-range indices N={n}")
        c = random_matrix(n, n, symmetric=True)
        perms = random_perms(n, 64, seed=n).astype(np.int32)
        perms[::3, 1] = 1 << 30
        perms[1::3, 2] = -7
        gpu_ring(c, perms, 0)
        if n & (n - 1) == 0:
            gpu_rd(c, perms)
        good = np.ones(64, dtype=bool)
        good[::3] = False
        good[1::3] = False
        assert np.array_equal(gpu_ring(c, perms, 0)[good], oracle.ring_cost_batch(c, perms[good], 0))


def test_validate_matrix():
    say("validate matrix")
    c = make_matrix(2)
    assert cc.cc_validate_matrix(dev(c), True) == 0
    a = make_matrix(3)
    assert cc.cc_validate_matrix(dev(a), True) == -5
    assert cc.cc_validate_matrix(dev(a), False) == 0
    bad = c.copy()
    bad[3, 5] = COST_MAX + 1
    assert cc.cc_validate_matrix(dev(bad), False) == -6
    bad[3, 5] = -1
    assert cc.cc_validate_matrix(dev(bad), False) == -6


@pytest.mark.parametrize("n", [2, 3, 31, 63, 64, 65, 100, 128, 129, 191, 192, 255, 256, 257, 500, 1024])
def test_init_tours_every_generation_path(n):
    """Seeded start orders for sizes on both sides of every switch of the generator (one node per lane, up to four per
    lane, the replay in LDS), with a first id above zero and a count that is no multiple of the launch shape."""
    say(f"cc_init_tours N={n}")
    seed, first, count = 0x5eed0000 + n, 1000003, 1037
    tours = cc.cc_init_tours(n, count, seed, first=first)
    torch.cuda.synchronize()
    assert np.array_equal(tours.cpu().numpy(), oracle.init_tours(seed, n, count, first=first))


def test_calls_on_an_explicit_stream_own_their_allocations():
    """The binding allocates outputs and workspaces for calls that only enqueue kernels; given a stream that is not
    torch's current one it must tell the allocator so (a dropped workspace may not be reused while the kernels still
    run).  Batches and a search on a side stream, with allocator churn on the current stream in between."""
    n = 256
    c = random_matrix(n, 41, symmetric=False, lo=0, hi=50000)
    perms = random_perms(n, 40000, 42)
    side = torch.cuda.Stream()
    cd, pd = dev(c), dev(perms)
    torch.cuda.synchronize()
    say("explicit stream: halving-doubling and BCube batches with binding-owned workspace, 2-opt search")
    rd = cc.cc_rd_cost_batch(cd, pd, stream=side)
    junk = [torch.full((1 << 18,), 7, dtype=torch.int32, device="cuda") for _ in range(8)]     # churn on the current stream
    bc = cc.cc_bcube_cost_batch(cd, 4, pd, stream=side)
    res = cc.cc_2opt_search_ex(dev(random_matrix(64, 43, True, 1, 9000)), 0, 64, 5, stream=side)
    junk += [torch.full((1 << 18,), 9, dtype=torch.int32, device="cuda") for _ in range(8)]
    side.synchronize()
    torch.cuda.synchronize()
    assert np.array_equal(rd.cpu().numpy(), oracle.rd_cost_batch(c, perms))
    assert np.array_equal(bc.cpu().numpy(), oracle.bcube_cost_batch(c, 4, perms))
    want = oracle.search(random_matrix(64, 43, True, 1, 9000), 0, 64, seed=5)
    assert np.array_equal(res.restart_costs.cpu().numpy(), want["costs"]) and int(res.best_cost.item()) == want["best_cost"]
    del junk
