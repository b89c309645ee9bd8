"""GPU parity of the logits pass on adversarial rows, through the C ABI: every row is the root
row of its own sequence (one layer, one frontier slot), so the candidate dump of the layer holds
the row's top-K token ids, probabilities and entropy, compared with the oracle's row definition."""
import numpy as np
import pytest
import torch

from _harness import RTOL, close, to_np

pytestmark = pytest.mark.gpu


def _bf16_round(x):
    return torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16)


def adversarial_rows(V, rng, bf16):
    rows, names = [], []

    def add(name, r):
        names.append(name); rows.append(np.asarray(r, np.float32))

    add("normal", 3 * rng.standard_normal(V))
    add("all_equal", np.full(V, 1.5))
    add("all_zero", np.zeros(V))
    oh = np.zeros(V); oh[V // 3] = 30.0
    add("one_hot", oh)
    oh2 = -5 + 0.01 * rng.standard_normal(V); oh2[V - 1] = 20.0
    add("spike_last", oh2)
    add("ties_coarse", np.round(2 * rng.standard_normal(V)))            # a handful of distinct values
    mi = 2 * rng.standard_normal(V); mi[rng.random(V) < 0.3] = -np.inf
    add("minus_inf_30pct", mi)
    mi9 = 2 * rng.standard_normal(V); mi9[rng.random(V) < 0.9] = -np.inf   # most chunks hold nothing but -inf
    add("minus_inf_90pct", mi9)
    mit = 2 * rng.standard_normal(V); mit[rng.random(V) < 0.2] = -np.inf; mit[rng.random(V) < 0.05] = 0.0
    mit[V - 1] = -np.inf; mit[V - 2] = 7.0                                # masked, zero and largest logits side by side
    add("minus_inf_with_zeros", mit)
    # large negative constants in place of -inf: e^(x - m) is exactly 0 in fp64 for them
    fm = 2 * rng.standard_normal(V); fm[rng.random(V) < 0.3] = -3.3895313892515355e38      # the lowest bf16
    add("masked_lowest_bf16", fm)
    f9 = 2 * rng.standard_normal(V); f9[rng.random(V) < 0.5] = -1e9; f9[rng.random(V) < 0.1] = -np.inf; f9[rng.random(V) < 0.05] = -1e4
    add("masked_mixed_constants", f9)
    nb = -118 + 1.5 * rng.standard_normal(V); nb[rng.random(V) < 0.1] = -1024.0     # the least negative masked value, lowest row maximum
    add("masked_minus_1024_low_row", nb)
    nb2 = 2 * rng.standard_normal(V); nb2[rng.random(V) < 0.01] = -1016.0         # just inside (-2^10, -2^7]: not masked, two-pass path
    add("minus_1016_not_masked", nb2)
    mi2 = np.full(V, -np.inf); mi2[[0, V // 2, V - 1]] = [1.0, 2.0, 2.0]
    add("only_three_finite", mi2)
    add("sorted_desc", np.sort(3 * rng.standard_normal(V))[::-1].copy())
    add("sorted_asc", np.sort(3 * rng.standard_normal(V)))
    add("all_negative_large", -1000 + rng.standard_normal(V))
    add("wide_range", 40 * rng.standard_normal(V))
    blk = 0.1 * rng.standard_normal(V); blk[:: 8 * 256] += 10.0           # maxima land in one lane's chunks
    add("strided_maxima", blk)
    add("signed_zeros", np.where(rng.random(V) < 0.5, -0.0, 0.0))
    zh = np.where(rng.random(V) < 0.5, -0.0, 0.0); zh[rng.choice(V, min(V, 48), replace=False)] = rng.uniform(1, 9, min(V, 48))
    add("zeros_with_positive_head", zh)                                  # below-window values inside the fast path
    tn = 3 * rng.standard_normal(V); tn[rng.random(V) < 0.01] = 1e-9; tn[rng.random(V) < 0.01] = -1e-12
    add("sprinkled_tiny", tn)
    # few positive logits, a few below-window ones, the rest negative: the M largest (M = 1000) then
    # take all positives, all below-window values and only some of the negative ones
    fp = -5 + rng.standard_normal(V); fp[rng.choice(V, min(V, 200), replace=False)] = rng.uniform(1, 5, min(V, 200))
    fp[rng.choice(V, min(V, 30), replace=False)] = rng.choice([0.0, -0.0, 1e-9, -1e-12], min(V, 30))
    add("few_positive_some_tiny", fp)
    lowhigh = -20 + rng.standard_normal(V); lowhigh[V // 2:] += 60       # reference must be raised mid-row
    add("late_large", lowhigh)
    if V > 70000:
        # one value held by exactly 65535 / 65536 logits: the largest count a 16-bit histogram
        # counter holds, and the smallest one that overflows it
        for n_same in (65535, 65536):
            r = 3 * rng.standard_normal(V); r[rng.choice(V, n_same, replace=False)] = -0.75
            add("same_value_%d" % n_same, r)
            r = 3 * rng.standard_normal(V); r[rng.choice(V, n_same, replace=False)] = 4.0   # ties reach the top K
            add("same_top_value_%d" % n_same, r)
    return names, np.stack(rows)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("V,K,splits", [(32000, 10, 0), (128256, 16, 0), (128256, 32, 5), (5003, 8, 0), (5003, 64, 3),
                                         (70, 64, 0), (152064, 32, 1), (152064, 32, 0), (49163, 16, 0), (65541, 16, 0)])
def test_rows_against_oracle(dtype, V, K, splits):
    from oracle import ref_row
    from paper_2502_13652_amd import C2TContext
    rng = np.random.default_rng(V * 31 + K)
    names, rows = adversarial_rows(V, rng, dtype == "bf16")
    B = rows.shape[0]
    epc = 8 if dtype == "bf16" else 4
    stride = (V + epc - 1) // epc * epc + epc          # padded stride; padding poisoned with +inf
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    x = torch.full((B, 1, stride), float("inf"), dtype=tdt)
    x[:, 0, :V] = torch.from_numpy(rows).to(tdt)
    xd = x.cuda()
    h = 2
    ctx = C2TContext(B, V, 1, K, 1, 1, h, 1 if dtype == "bf16" else 0, 0.0)
    W1 = np.zeros((h, 3), np.float32); W1[0, 0] = 1
    ctx.set_classifier(W1, np.zeros(h, np.float32), np.array([1, 0], np.float32), 0.0)
    if splits:
        from paper_2502_13652_amd import C2TError
        while True:                      # a split count whose cell map does not fit the LDS is refused: take the fewest that fit
            try:
                ctx.set_row_splits(splits, splits)
                break
            except C2TError as e:
                assert e.code == -2 and splits < 16
                splits += 1
    if dtype == "bf16" and splits == 0:
        # long rows, few of them: several workgroups count one row and add their histograms up.  49163 and
        # 65541 logits: the last of them gets two chunks (one partial) / nothing but the row's partial chunk
        want = {128256: 4, 152064: 5, 49163: 4, 65541: 5}.get(V, 1)
        assert B <= 256 // want and ctx.row_workgroups() == (want, want), ctx.row_workgroups()
    print("rows V=%d K=%d %s splits=%d" % (V, K, dtype, splits), flush=True)
    ctx.reset()
    ctx.expand_layer(xd)
    torch.cuda.synchronize()
    c = to_np(ctx.candidates())
    status = to_np(ctx.finalize_tree())["status"]
    if dtype == "bf16" and V >= 5003:
        # masked logits (-inf, large negative constants) do not push a row off the histogram path
        for b, name in enumerate(names):
            if name.startswith("masked_") or name in ("minus_inf_30pct", "minus_inf_90pct", "minus_inf_with_zeros", "normal"):
                assert not status[b] & 2, name
            if name in ("minus_1016_not_masked", "wide_range"):
                assert status[b] & 2, name
    xin = x[:, 0, :V].contiguous()
    bits = xin.view(torch.int16).numpy().view(np.uint16) if dtype == "bf16" else xin.numpy()
    for b, name in enumerate(names):
        r = ref_row(bits[b], K)
        assert not r["bad"], name
        k = len(r["ids"])
        np.testing.assert_array_equal(c["token"][b, :k], r["ids"], err_msg=name)
        ok = close(c["p"][b, :k], r["p"].astype(np.float32), atol=1e-37)
        assert ok.all(), "%s p: %s vs %s" % (name, c["p"][b, :k][~ok][:3], r["p"][~ok][:3])
        # absolute floor: the oracle adds V terms one by one in fp64, so its Z (and with it H = ln Z - S/Z)
        # carries up to V * 2^-53 of rounding; only rows with H below ~1e-5 ever get near it
        assert close(c["H"][b, 0], np.float32(r["H"]), atol=V * 2.0 ** -53).all(), "%s H: %g vs %g" % (name, c["H"][b, 0], r["H"])
        assert (c["z"][b, :k] == c["P"][b, :k]).all() and (c["P"][b, :k] == c["p"][b, :k]).all()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("V,M,splits", [(32000, 1000, 0), (128256, 1000, 0), (5003, 1, 0), (5003, 37, 0), (5003, 5003, 0), (70, 1000, 0),
                                         (5003, 37, 3), (32000, 1000, 7), (152064, 1000, 0), (5003, 6000, 2), (65541, 3000, 0)])
def test_entropy_over_the_top_m_against_oracle(dtype, V, M, splits):
    # Eq. 2, second line: H over the M most probable tokens of the full softmax
    from oracle import ref_entropy_top_m, ref_row
    from paper_2502_13652_amd import C2TContext
    rng = np.random.default_rng(V * 7 + M)
    names, rows = adversarial_rows(V, rng, dtype == "bf16")
    B, K = rows.shape[0], 4
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    x = torch.from_numpy(rows).to(tdt).view(B, 1, V)
    if V % 8:
        xp = torch.full((B, 1, (V + 7) // 8 * 8), float("inf"), dtype=tdt); xp[:, :, :V] = x; x = xp
    # fp32 rows of more than 49152 logits are split by the library itself; `splits` forces it elsewhere
    ctx = C2TContext(B, V, 1, K, 1, 1, 2, 1 if dtype == "bf16" else 0, 0.0, entropy_top_m=M)
    if splits:
        ctx.set_row_splits(splits, splits)
    W1 = np.zeros((2, 3), np.float32); W1[0, 0] = 1
    ctx.set_classifier(W1, np.zeros(2, np.float32), np.array([1, 0], np.float32), 0.0)
    print("top-M entropy V=%d M=%d %s splits=%d" % (V, M, dtype, splits), flush=True)
    ctx.reset()
    ctx.expand_layer(x.cuda())
    torch.cuda.synchronize()
    c = to_np(ctx.candidates())
    xin = x[:, 0, :V].contiguous()
    bits = xin.view(torch.int16).numpy().view(np.uint16) if dtype == "bf16" else xin.numpy()
    for b, name in enumerate(names):
        HM = ref_entropy_top_m(bits[b], M)
        full = ref_row(bits[b], 1)["H"]
        assert close(c["H"][b, 0], np.float32(HM), atol=V * 2.0 ** -53).all(), "%s H_M: %g vs %g (full %g)" % (name, c["H"][b, 0], HM, full)
        if M >= V:
            assert close(c["H"][b, 0], np.float32(full), atol=V * 2.0 ** -53).all(), name


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_bad_rows_set_status_and_yield_nothing(dtype):
    from paper_2502_13652_amd import C2TContext
    V, K = 4096 + 8, 4
    rng = np.random.default_rng(5)
    rows = (2 * rng.standard_normal((5, V))).astype(np.float32)
    rows[1, 777] = np.nan
    rows[2, V - 1] = np.inf
    rows[3, :] = -np.inf
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    x = torch.from_numpy(rows).to(tdt).view(5, 1, V).cuda()
    ctx = C2TContext(5, V, 1, K, 1, 4, 2, 1 if dtype == "bf16" else 0, 0.0)
    W1 = np.zeros((2, 3), np.float32); W1[0, 0] = 1
    ctx.set_classifier(W1, np.zeros(2, np.float32), np.array([1, 0], np.float32), 0.0)
    for splits in (1, 2):
        ctx.set_row_splits(splits, splits)
        ctx.reset()
        ctx.expand_layer(x)
        out = to_np(ctx.finalize_tree())
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out["status"] & 1, [0, 1, 1, 1, 0])
        np.testing.assert_array_equal(out["n_nodes"], [1, 0, 0, 0, 1])
        assert (out["tokens"][1:4] == -1).all() and not out["mask"][1:4].any()
