"""gram_unique_static, the dedup entry point that allocates nothing (its scratch memory is a
fixed array in the library's device image), against gram_unique through the C ABI: bit-exact
outputs on calls in a row that share the one array, the later ones with smaller inputs."""
import numpy as np
import pytest

from paper_2204_04179_amd import workloads as wl

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def zipf_ids(m, n, seed, pad_frac=0.1):
    rng = np.random.default_rng(seed)
    p = 1.0 / np.arange(1, n, dtype=np.float64) ** 1.05
    cdf = np.cumsum(p)
    r = np.searchsorted(cdf, rng.random(m) * cdf[-1])
    ids = (rng.permutation(n - 1)[np.minimum(r, n - 2)] + 1).astype(np.int32)
    ids[rng.random(m) < pad_frac] = 0
    return ids


def both_ways(torch, gram, ids_np, n, pad_id):
    """(uniq, inverse, counts, U) from gram_unique on a context, and from gram_unique_static."""
    m = ids_np.size
    cap = max(1, min(m, n))
    i32 = dict(dtype=torch.int32, device="cuda")
    ids = torch.from_numpy(ids_np).cuda()

    def buffers():
        return (torch.full((cap,), -7, **i32), torch.full((max(1, m),), -7, **i32), torch.full((cap,), -7, **i32),
                torch.full((1,), -7, **i32))

    g = gram.Gram(gram.make_config(n, 8, 4, max(1, m), 1, pad_id, 0, gram.F32))
    uq, inv, cnt, u = buffers()
    U = g.unique(ids, uq, inv, cnt, u, want_host_u=True)
    g.close()
    uq2, inv2, cnt2, u2 = buffers()
    err = torch.full((1,), -7, **i32)
    gram.unique_static(ids, n, pad_id, uq2, inv2, cnt2, u2, err, m=m)
    torch.cuda.synchronize()
    U2 = int(u2.item())
    ref = (uq[:U].cpu().numpy(), inv[:m].cpu().numpy(), cnt[:U].cpu().numpy(), U)
    got = (uq2[:U2].cpu().numpy(), inv2[:m].cpu().numpy(), cnt2[:U2].cpu().numpy(), U2)
    tail_untouched = bool((uq2[U2:] == -7).all().item()) and bool((cnt2[U2:] == -7).all().item())
    return ref, got, int(err.item()), tail_untouched


def test_unique_without_allocation_matches_gram_unique_on_calls_in_a_row():
    import torch
    from paper_2204_04179_amd import gram
    n = 1_000_000
    # the stress batch shape (multi-kernel sort, two radix passes), then smaller inputs that reuse
    # the same static array: a mid-size batch, a one-launch batch, one position, none
    for m, seed in ((204_800, 1), (20_001, 2), (5_000, 3), (1, 4), (0, 5), (gram.UNIQUE_STATIC_MAX_POSITIONS, 6),
                    (8_193, 7)):
        ids = zipf_ids(m, n, seed) if m else np.zeros(0, np.int32)
        ref, got, err, tail = both_ways(torch, gram, ids, n, 0)
        say(f"static unique m={m}: U={ref[3]}")
        assert got[3] == ref[3]
        for a, b in zip(ref[:3], got[:3]):
            np.testing.assert_array_equal(a, b)
        assert err == 0 and tail
        if m:
            u, inv, cnt = np.unique(ids, return_inverse=True, return_counts=True)
            np.testing.assert_array_equal(got[0], u)
            np.testing.assert_array_equal(got[1], inv)
            np.testing.assert_array_equal(got[2], cnt)


def test_unique_without_allocation_small_vocabulary_and_other_padding_ids():
    import torch
    from paper_2204_04179_amd import gram
    rng = np.random.default_rng(9)
    for n, m, pad in ((50, 30_000, 0), (300, 9_000, -1), (2, 70_000, 1), (1 << 24, 100_000, 7)):
        ids = rng.integers(0, n, size=m).astype(np.int32)
        ref, got, err, tail = both_ways(torch, gram, ids, n, pad)
        say(f"static unique n={n} m={m} pad={pad}: U={ref[3]}")
        assert got[3] == ref[3] and err == 0 and tail
        for a, b in zip(ref[:3], got[:3]):
            np.testing.assert_array_equal(a, b)


def test_unique_without_allocation_reports_errors():
    import torch
    from paper_2204_04179_amd import gram
    i32 = dict(dtype=torch.int32, device="cuda")
    n = 1000
    # an ID outside [0, N) is flagged on the device and counted as the padding ID
    for m in (3_000, 40_000):
        ids = np.random.default_rng(m).integers(1, n, size=m).astype(np.int32)
        ids[17], ids[m - 1] = n + 5, -3
        fixed = ids.copy()
        fixed[[17, m - 1]] = 0
        uq, cnt, inv = torch.zeros(n, **i32), torch.zeros(n, **i32), torch.zeros(m, **i32)
        u, err = torch.zeros(1, **i32), torch.zeros(1, **i32)
        gram.unique_static(torch.from_numpy(ids).cuda(), n, 0, uq, inv, cnt, u, err)
        torch.cuda.synchronize()
        assert int(err.item()) == 1
        ref_u, ref_inv, ref_cnt = np.unique(fixed, return_inverse=True, return_counts=True)
        U = int(u.item())
        assert U == ref_u.size
        np.testing.assert_array_equal(uq[:U].cpu().numpy(), ref_u)
        np.testing.assert_array_equal(inv.cpu().numpy(), ref_inv)
        np.testing.assert_array_equal(cnt[:U].cpu().numpy(), ref_cnt)
        # the next call starts from a clean flag
        ok = torch.from_numpy(fixed).cuda()
        gram.unique_static(ok, n, 0, uq, inv, cnt, u, err)
        torch.cuda.synchronize()
        assert int(err.item()) == 0
    # sizes beyond the fixed maximum and bad arguments are refused on the host
    big = torch.zeros(gram.UNIQUE_STATIC_MAX_POSITIONS + 1, **i32)
    out = torch.zeros(big.numel(), **i32)
    u = torch.zeros(1, **i32)
    with pytest.raises(gram.GramError) as e:
        gram.unique_static(big, n, 0, out, out, out, u)
    assert e.value.status == gram.ERR_CAPACITY and "maximum" in str(e.value)
    with pytest.raises(gram.GramError) as e:
        gram.unique_static(big[:10], n, 0, out, out, out, None)
    assert e.value.status == gram.ERR_ARG
    with pytest.raises(gram.GramError) as e:
        gram.unique_static(big[:10], 0, 0, out, out, out, u)
    assert e.value.status == gram.ERR_ARG
