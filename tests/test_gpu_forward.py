"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2511_00101_amd import binding as lq
from paper_2511_00101_amd import synth

from gpu_util import (long_batch_problem, DeviceProblem, assert_close, assert_tables_equal, check_forward,
                      check_forward_group, group_of)

pytestmark = pytest.mark.gpu

VARIANTS = [lq.LQ_VARIANT_SPLIT, lq.LQ_VARIANT_FUSED, lq.LQ_VARIANT_SLAB, lq.LQ_VARIANT_AUTO]


# ---------------------------------------------------------------------------------------------------
# segment metadata: bit exact
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("T,n_ad", [(0, 3), (1, 1), (63, 4), (64, 4), (65, 7), (200, 300), (256, 64), (257, 64), (1000, 64), (2047, 9), (2048, 16), (2049, 5),
                                    (4097, 33), (8192, 32), (16385, 40), (5000, 300), (5000, 313), (20000, 1000),
                                    (140000, 24)])
def test_build_segments_bit_exact(oracle_mod, T, n_ad):
    rng = np.random.default_rng(T * 131 + n_ad)
    ranks = rng.integers(1, 65, size=n_ad).astype(np.int32)
    ta = rng.integers(-1, n_ad + 1, size=T).astype(np.int32)       # includes -1 and one id beyond the table
    tk = rng.integers(0, 4, size=T).astype(np.uint8)               # includes one unknown kind
    if T > 100:  # long runs as well as scattered tokens
        ta[: T // 3] = 1 % n_ad
        tk[: T // 3] = 0
    ref = oracle_mod.build_segments(ta, tk, ranks)
    seg = lq.SegmentTables.empty(T, n_ad)
    ws = lq.workspace(lq.lora_build_workspace_bytes(T, n_ad))
    lq.lora_build_segments(torch.from_numpy(ta).cuda(), torch.from_numpy(tk).cuda(), torch.from_numpy(ranks).cuda(),
                           seg, ws)
    assert_tables_equal(seg.to_host(), ref)


def test_build_segments_one_and_many_workgroups_agree(oracle_mod):
    """Batches of 2048 tokens and more are built by several workgroups when a workspace is given and by one
    without; both must give the oracle's tables, also when the same workspace is used again and again."""
    rng = np.random.default_rng(77)
    T, n_ad = 8192 + 37, 48
    ranks = rng.integers(1, 65, size=n_ad).astype(np.int32)
    ws = lq.workspace(lq.lora_build_workspace_bytes(T, n_ad))
    for rep in range(3):
        ta = rng.integers(-1, n_ad + 1, size=T).astype(np.int32)
        tk = rng.integers(0, 4, size=T).astype(np.uint8)
        ta[rep * 1000: rep * 1000 + 3000] = rep       # a long run that straddles workgroup boundaries
        tk[rep * 1000: rep * 1000 + 3000] = rep % 3
        ref = oracle_mod.build_segments(ta, tk, ranks)
        d_ta, d_tk, d_r = torch.from_numpy(ta).cuda(), torch.from_numpy(tk).cuda(), torch.from_numpy(ranks).cuda()
        for workspace in (ws, None):
            seg = lq.SegmentTables.empty(T, n_ad)
            lq.lora_build_segments(d_ta, d_tk, d_r, seg, workspace)
            assert_tables_equal(seg.to_host(), ref)
    assert int(ws[0].item() & 0xffffffff) == 0


def test_build_segments_configs(oracle_mod):
    for p in (synth.config1(), synth.config2()):
        d = DeviceProblem(p)
        d.build()
        assert_tables_equal(d.seg.to_host(), oracle_mod.build_segments(p.batch.token_adapter, p.batch.token_kind, p.ranks))
    for b, n_ad, ranks in ((synth.batch_unified(np.random.default_rng(3500)), 32, [16] * 32),
                           (synth.batch_zipf(np.random.default_rng(4500)), 32, [(8, 16, 32, 64)[i % 4] for i in range(32)]),
                           (synth.config5_batch(), 16, [32] * 16)):
        ranks = np.asarray(ranks, np.int32)
        seg = lq.SegmentTables.empty(b.n_tokens, n_ad)
        lq.lora_build_segments(torch.from_numpy(b.token_adapter).cuda(), torch.from_numpy(b.token_kind).cuda(),
                               torch.from_numpy(ranks).cuda(), seg, lq.workspace(lq.lora_build_workspace_bytes(b.n_tokens, n_ad)))
        assert_tables_equal(seg.to_host(), oracle_mod.build_segments(b.token_adapter, b.token_kind, ranks))


# ---------------------------------------------------------------------------------------------------
# forward: element by element against the oracle
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("y0_zero", [False, True])
def test_config1_tiny(oracle_mod, variant, y0_zero):
    check_forward(oracle_mod, synth.config1(y0_zero=y0_zero), variant)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("seed,T,d_in,d_out,ranks", [
    (1, 37, 520, 264, [1, 3, 8, 64]),           # d not a multiple of the 512-wide wave tile, odd ranks
    (2, 300, 1032, 776, [16, 128, 5, 24, 33]),  # several tiles, ragged tails, maximum rank
    (3, 5, 8, 8, [2]),                           # smallest supported shape
    (4, 130, 2048, 4096, [8, 16, 32]),
])
def test_small_mixed(oracle_mod, variant, seed, T, d_in, d_out, ranks):
    for y0_zero in (False, True):
        p = synth.small_mixed(seed, T, d_in, d_out, ranks, drop_frac=0.1, y0_zero=y0_zero, w_std=0.05)
        check_forward(oracle_mod, p, variant)


@pytest.mark.parametrize("variant", VARIANTS)
def test_zero_B_is_bit_identical(oracle_mod, variant):
    p = synth.small_mixed(9, 77, 512, 512, [8, 16], drop_frac=0.2)
    p.B = [np.zeros_like(b) for b in p.B]
    d = DeviceProblem(p)
    d.build()
    y_bits, _, err = d.forward(variant)
    assert err == 0 and np.array_equal(y_bits, p.y0)


@pytest.mark.parametrize("variant", VARIANTS)
def test_identity_perm_with_caller_tables(oracle_mod, variant):
    """Tables written by the caller for a batch that is already in segment order, perm = NULL."""
    rng = np.random.default_rng(17)
    lens, ads, kinds = [70, 3, 1, 20], [2, 0, 1, 0], [0, 1, 2, 2]
    ta = np.concatenate([np.full(l, a, np.int32) for l, a in zip(lens, ads)])
    tk = np.concatenate([np.full(l, k, np.uint8) for l, k in zip(lens, kinds)])
    p = synth.make_problem("sorted", synth.Batch(ta, tk), 256, 384, [8, 4, 16], [1.0, 2.0, 0.5], 99)
    ref = oracle_mod.forward(p.x, p.y0, p.A, p.B, p.ranks, p.scales, ta, tk)
    d = DeviceProblem(p)
    seg = d.seg
    seg.seg_starts[:5] = torch.tensor(np.cumsum([0] + lens), dtype=torch.int32)
    seg.seg_adapter[:4] = torch.tensor(ads, dtype=torch.int32)
    seg.seg_kind[:4] = torch.tensor(kinds, dtype=torch.uint8)
    seg.h_offsets[:5] = torch.tensor([0, 70 * 16, 70 * 16, 70 * 16, 70 * 16], dtype=torch.int64)
    seg.n_segments[0] = 4
    y_bits, h, err = d.forward(variant, h_elems=70 * 16, use_perm=False)
    assert err == 0
    assert_close(synth.bf16_bits_to_f64(y_bits), ref.y, "y")
    assert_close(h, ref.h, "h")


@pytest.mark.parametrize("variant", VARIANTS)
def test_bad_device_metadata_is_skipped_and_flagged(variant):
    p = synth.small_mixed(23, 40, 256, 256, [8, 8], n_kinds=1)
    d = DeviceProblem(p)
    d.build()
    d.seg.seg_adapter[0] = 7                    # beyond the adapter table
    y_bits, _, err = d.forward(variant)
    assert err & 1
    rows = d.seg.to_host()
    first = rows["perm"][rows["seg_starts"][0]: rows["seg_starts"][1]]
    assert np.array_equal(y_bits[first], p.y0[first])
    # the binding's checked mode turns the word into an exception
    word = torch.tensor([err], dtype=torch.int32, device="cuda")
    with pytest.raises(lq.LqDeviceError, match="bad segment"):
        lq.raise_on_device_error(word, "forward")
    lq.raise_on_device_error(torch.zeros(1, dtype=torch.int32, device="cuda"))   # a clean word raises nothing


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("corrupt", ["start_negative", "end_beyond_batch", "runs_backwards"])
def test_corrupt_segment_range_is_skipped_and_flagged(oracle_mod, variant, corrupt):
    """A segment whose positions leave [0, n_tokens] or run backwards (tables written by a careless caller) is
    treated as empty and reported; every other segment is computed as usual and nothing is accessed out of
    bounds (the guard clamps before any index is formed)."""
    lens, ads, kinds = [40, 50, 6], [0, 1, 0], [0, 1, 2]
    ta = np.concatenate([np.full(l, a, np.int32) for l, a in zip(lens, ads)])
    tk = np.concatenate([np.full(l, k, np.uint8) for l, k in zip(lens, kinds)])
    p = synth.make_problem("corrupt", synth.Batch(ta, tk), 256, 256, [8, 16], [1.0, 2.0], 5)
    ref = oracle_mod.forward(p.x, p.y0, p.A, p.B, p.ranks, p.scales, ta, tk)
    d = DeviceProblem(p)
    d.build()
    starts = d.seg.seg_starts.cpu().numpy().copy()      # [0, 40, 90, 96]
    if corrupt == "start_negative":
        starts[0] = -5                                   # segment 0 = [-5, 40)
        bad = [0]
    elif corrupt == "end_beyond_batch":
        starts[3] = 96 + 1000                            # segment 2 = [90, 1096)
        bad = [2]
    else:
        starts[2] = 30                                   # segment 1 = [40, 30) runs backwards; segment 2 = [30, 96) is a
        bad = [1]                                        # valid range that now overlaps others: only rows 0..29 are compared
    d.seg.seg_starts[:4] = torch.from_numpy(starts[:4]).cuda()
    y_bits, _, err = d.forward(variant, h_elems=40 * 8)
    assert err & 1
    y = synth.bf16_bits_to_f64(y_bits)
    if corrupt == "runs_backwards":
        assert_close(y[:30], ref.y[:30], "rows of segment 0 that no other segment touches")
        return
    bounds = [0, 40, 90, 96]
    for g in range(3):
        rows = slice(bounds[g], bounds[g + 1])
        if g in bad:
            assert np.array_equal(y_bits[rows], p.y0[rows])           # skipped: untouched
        else:
            assert_close(y[rows], ref.y[rows], f"segment {g}")


@pytest.mark.parametrize("variant", VARIANTS)
def test_config2_decode_heavy(oracle_mod, variant):
    for y0_zero in (False, True):
        check_forward(oracle_mod, synth.config2(y0_zero=y0_zero), variant)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("y0_zero", [False, True])
def test_config3_unified(oracle_mod, variant, y0_zero):
    check_forward(oracle_mod, synth.config3(y0_zero=y0_zero), variant)


def request_scales(p, seed):
    """A per-token scale as per-request dynamic scaling would produce it: runs of tokens (requests) share a value,
    different requests of the same adapter differ; some are negative, some zero."""
    rng = np.random.default_rng(seed)
    ts = np.empty(p.n_tokens, np.float32)
    t = 0
    while t < p.n_tokens:
        n = int(rng.integers(1, 40))
        ts[t: t + n] = rng.choice([0.0, 0.25, -0.5, 1.0, 1.5, 2.0, 3.0])
        t += n
    return ts


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("y0_zero", [False, True])
def test_dynamic_per_token_scale(oracle_mod, variant, y0_zero):
    """Section 3.3's dynamic scaling: token_scales replaces the per-adapter scale row by row, in the short (decode)
    units and in the long (MFMA) ones, with and without a k split; the saved h stays unscaled."""
    for p in (synth.small_mixed(51, 300, 1032, 776, [16, 128, 5, 24, 33], drop_frac=0.1, y0_zero=y0_zero, w_std=0.03),   # (|y| stays below 8)
              synth.config2(y0_zero=y0_zero), synth.config3(y0_zero=y0_zero)):
        p.scales = np.full_like(p.scales, 1000.0)       # must be ignored
        check_forward(oracle_mod, p, variant, token_scales=request_scales(p, 7))


# ---------------------------------------------------------------------------------------------------
# grouped call: several linear layers that read the same x (Algorithm 1: Q, K, V from one X)
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("n_proj", [1, 2, 3, 4])
def test_group_small_mixed(oracle_mod, variant, n_proj):
    """Ragged shapes, ranks 3..128, rows without adapter; every layer of the group against the oracle's result for
    that layer alone; also with the dynamic per-token scale."""
    base = synth.small_mixed(71, 300, 1032, 776, [16, 128, 5, 24, 33], drop_frac=0.1, w_std=0.03)
    group = group_of(base, [264, 1544, 8][: n_proj - 1], 700)
    check_forward_group(oracle_mod, group, variant)
    if n_proj == 3:
        check_forward_group(oracle_mod, group, variant, token_scales=request_scales(base, 11))


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("ranks,n_tokens", [([16, 7, 12], 700), ([32, 20, 3, 17], 6000), ([64, 40, 33], 700)])
def test_group_of_four_by_rank_class(oracle_mod, variant, ranks, n_tokens):
    """Four layers in one call at ranks up to 16, 32 and 64: the slab kernel keeps the accumulators of four, three
    and one projection(s) per pass, so these run as one pass, as 3 + 1 and as 1 + 1 + 1 + 1; 700 tokens give slabs of
    one 16-row tile, 6000 tokens slabs of two; saved h per layer."""
    base = synth.small_mixed(171, n_tokens, 520, 264, ranks, drop_frac=0.05, w_std=0.03)
    check_forward_group(oracle_mod, group_of(base, [1032, 8, 776], 1700), variant)


@pytest.mark.parametrize("variant", VARIANTS)
def test_group_unified_batch(oracle_mod, variant):
    """Long fine-tune segments with a k split, prefill and decode segments, saved h per layer."""
    base = synth.config3()
    check_forward_group(oracle_mod, group_of(base, [1024, 2048], 800), variant)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("which", ["qkv", "gate_up"])
def test_group_layer_stack_shapes(oracle_mod, variant, which):
    """The two groups of the layer stack at full size: q, k, v (4096 -> 4096, 1024, 1024) and gate, up (4096 -> 14336)."""
    if which == "qkv":
        group = group_of(synth.config5(3, 0, with_dy=False), [1024, 1024], 900)
    else:
        group = group_of(synth.config5(3, 4, with_dy=False), [14336], 910)
    check_forward_group(oracle_mod, group, variant)


def test_group_rejects_bad_arguments():
    p = synth.config1()
    d = DeviceProblem(p)
    d.build()
    ws = lq.workspace(lq.lora_forward_group_workspace_bytes(2, p.n_tokens, 8))
    y2 = d.y.clone()
    with pytest.raises(lq.LqError) as e:
        lq.lora_segmented_forward_group(d.x, [d.y, d.y], [d.adapters, d.adapters], d.seg, None, ws)     # the same y twice
    assert e.value.status == lq.LQ_ERR_INVALID_ARG
    small = lq.workspace(lq.lora_forward_group_workspace_bytes(1, p.n_tokens, 8))
    if small.numel() < ws.numel():
        with pytest.raises(lq.LqError) as e:
            lq.lora_segmented_forward_group(d.x, [d.y, y2], [d.adapters, d.adapters], d.seg, None, small)
        assert e.value.status == lq.LQ_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert np.array_equal(lq.bits_from_bf16(d.y), p.y0)


@pytest.mark.parametrize("variant", VARIANTS)
def test_repeat_calls_are_bit_identical(variant):
    p = synth.config2()
    outs = []
    for _ in range(3):
        d = DeviceProblem(p)
        d.build()
        outs.append(d.forward(variant)[0])
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


# ---------------------------------------------------------------------------------------------------
# full-size workloads in the launch configuration the benchmark times
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("which", ["up", "down"])
def test_config4_mlp_hetero_ranks(oracle_mod, variant, which):
    check_forward(oracle_mod, synth.config4(which), variant)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("which", ["up", "down"])
def test_config4_lora_term_alone(oracle_mod, variant, which):
    """y0 = 0, so the bound applies to the LoRA term itself and not to y0 + term."""
    check_forward(oracle_mod, synth.config4(which, y0_zero=True), variant)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("y0_zero", [False, True])
@pytest.mark.parametrize("layer,projection", [(0, 0), (0, 1), (31, 4), (31, 6)])
def test_config5_layer_stack_calls(oracle_mod, layer, projection, y0_zero, variant):
    """The four distinct shapes of the 224 (layer, projection) calls of the layer stack (q and k of layer 0, gate
    and down of layer 31), each in both variants, with y0 ~ N(0, 1) and with y0 = 0 (the LoRA term alone)."""
    check_forward(oracle_mod, synth.config5(layer, projection, with_dy=False, y0_zero=y0_zero), variant)


def test_large_rank_and_many_segments(oracle_mod):
    """Ranks up to the maximum and more than 128 segments (beyond the register-cached part of the tables)."""
    rng = np.random.default_rng(5)
    n_ad = 150
    ranks = rng.choice([4, 16, 40, 96, 128], size=n_ad)
    lens = rng.choice([1, 2, 3, 17, 40, 70, 130], size=n_ad)
    ta = np.concatenate([np.full(l, a, np.int32) for a, l in enumerate(lens)])
    tk = np.concatenate([np.full(l, a % 3, np.uint8) for a, l in enumerate(lens)])
    order = rng.permutation(len(ta))
    # weights and scales small enough that |y| stays below 8: from there on half a bf16 ulp of the output
    # alone (2^-5) exceeds the absolute bound
    for y0_zero in (False, True):
        p = synth.make_problem("many", synth.Batch(ta[order], tk[order]), 1024, 1536, ranks, rng.uniform(0.5, 1.0, n_ad), 321,
                               w_std=0.03, y0_zero=y0_zero)
        for variant in VARIANTS:
            check_forward(oracle_mod, p, variant)


@pytest.mark.parametrize("y0_zero", [False, True])
def test_many_tokens(oracle_mod, y0_zero):
    p = long_batch_problem(900, with_dy=False, y0_zero=y0_zero)
    for variant in VARIANTS:
        check_forward(oracle_mod, p, variant)


@pytest.mark.parametrize("variant", VARIANTS)
def test_token_permutation_invariance(oracle_mod, variant):
    """The update is per token, so the order of the tokens in the batch must not matter: permute the tokens, run the
    HIP path on the permuted batch, undo the permutation, and compare with the oracle's result for the ORIGINAL
    batch (y within tolerance; saved h through its own offsets; rows without an adapter bit-identical)."""
    p = synth.small_mixed(41, 700, 1032, 776, [16, 8, 33, 24], drop_frac=0.1, w_std=0.04)
    ref = oracle_mod.forward(p.x, p.y0, p.A, p.B, p.ranks, p.scales, p.batch.token_adapter, p.batch.token_kind)
    rng = np.random.default_rng(4242)
    for _ in range(2):
        sigma = rng.permutation(p.n_tokens)                      # row i of the permuted batch is token sigma[i]
        q = synth.Problem(p.name + "_perm", p.d_in, p.d_out, p.ranks, p.scales, p.A, p.B, p.x[sigma], p.y0[sigma],
                          synth.Batch(p.batch.token_adapter[sigma], p.batch.token_kind[sigma]))
        d = DeviceProblem(q)
        d.build()
        tables = d.seg.to_host()
        y_bits, h, err = d.forward(variant)
        assert err == 0
        back = np.empty_like(sigma)
        back[sigma] = np.arange(p.n_tokens)
        y_unperm = y_bits[back]
        assert_close(synth.bf16_bits_to_f64(y_unperm), ref.y, "y of the permuted batch, un-permuted")
        dead = p.batch.token_adapter < 0
        assert np.array_equal(y_unperm[dead], p.y0[dead])
        # saved h: token t's row sits where the permuted batch's own tables put it; its values are token t's
        ref_off = oracle_mod.token_h_offsets(ref.segments, p.ranks, p.n_tokens)
        for g in range(tables["n_segments"]):
            if tables["seg_kind"][g] != 0:
                continue
            r = int(p.ranks[tables["seg_adapter"][g]])
            rows = tables["perm"][tables["seg_starts"][g]: tables["seg_starts"][g + 1]]
            got = h[tables["h_offsets"][g]: tables["h_offsets"][g] + len(rows) * r].reshape(len(rows), r)
            want = np.stack([ref.h[ref_off[sigma[i]]: ref_off[sigma[i]] + r] for i in rows])
            assert_close(got, want, f"h of segment {g}")


def test_launch_timing_api():
    """lora_profile_enable / lora_profile_read: one record per launch, plausible durations, nothing left after a read."""
    p = synth.config1()
    d = DeviceProblem(p)
    lq.lora_profile_enable(True)
    try:
        for _ in range(3):
            d.build()
            d.forward(lq.LQ_VARIANT_SPLIT)
        d.forward(lq.LQ_VARIANT_FUSED)
        prof = lq.lora_profile_read()
        assert prof["build"][1] == 3 and prof["shrink"][1] == 3 and prof["expand"][1] == 3 and prof["forward_fused"][1] == 1
        for name in ("build", "shrink", "expand", "forward_fused"):
            total, n = prof[name]
            assert 0.5 < total / n < 1000.0, (name, total, n)   # microseconds
        assert all(n == 0 for _, n in lq.lora_profile_read().values())
    finally:
        lq.lora_profile_enable(False)
    d.forward(lq.LQ_VARIANT_SPLIT)
    assert all(n == 0 for _, n in lq.lora_profile_read().values())


def test_prepared_calls_match_direct_calls(oracle_mod):
    """binding.prepare_*: the same entry points with the arguments marshalled once."""
    p = synth.config1()
    direct, prepared = DeviceProblem(p), DeviceProblem(p)
    direct.build()
    y_direct, h_direct, _ = direct.forward(lq.LQ_VARIANT_FUSED)
    h_elems = int(direct.seg.h_offsets.max().item())
    prepared.h_out = torch.full((max(h_elems, 1),), float("nan"), dtype=torch.float32, device="cuda")
    ws = lq.workspace(lq.lora_forward_workspace_bytes(p.n_tokens, prepared.adapters.max_rank, p.d_in, p.d_out, lq.LQ_VARIANT_FUSED))
    build = lq.prepare_build_segments(prepared.token_adapter, prepared.token_kind, prepared.adapters.ranks, prepared.seg,
                                      prepared.build_ws)
    forward = lq.prepare_forward(prepared.x, prepared.y, prepared.adapters, prepared.seg, prepared.h_out, ws, lq.LQ_VARIANT_FUSED)
    build()
    forward()
    torch.cuda.synchronize()
    assert_tables_equal(prepared.seg.to_host(), oracle_mod.build_segments(p.batch.token_adapter, p.batch.token_kind, p.ranks))
    assert np.array_equal(lq.bits_from_bf16(prepared.y), y_direct)
    assert np.array_equal(prepared.h_out[:h_elems].cpu().numpy(), h_direct)


def test_fused_wait_that_runs_out_leaves_y_untouched(oracle_mod):
    """The single-launch variant's device-wide wait is bounded.  Here it can never complete (one arrival counter of
    the workspace header is pre-loaded with a large negative value by the host), so every workgroup's wait runs out:
    every kernel still exits normally, bit 1 of the error word is set, and y is bit-identical to y0 because the
    expand phase is skipped.  The same workspace keeps refusing single-launch calls until its header is zeroed;
    after that (or in two launches) the call gives the oracle's result."""
    p = synth.config1()
    ref = oracle_mod.forward(p.x, p.y0, p.A, p.B, p.ranks, p.scales, p.batch.token_adapter, p.batch.token_kind)
    d = DeviceProblem(p)
    d.build()
    ws = lq.workspace(lq.lora_forward_workspace_bytes(p.n_tokens, d.adapters.max_rank, p.d_in, p.d_out, lq.LQ_VARIANT_FUSED))
    words = ws.view(torch.int32)
    words[96] = -(1 << 20)                          # first arrival counter (header word 96)
    h_out = torch.zeros(ref.segments.h_elems, dtype=torch.float32, device="cuda")
    for _ in range(2):                              # the second call finds the poisoned generation word at once
        lq.lora_segmented_forward(d.x, d.y, d.adapters, d.seg, h_out, ws, lq.LQ_VARIANT_FUSED)
        torch.cuda.synchronize()
        assert int(words[0].item()) & 2
        assert np.array_equal(lq.bits_from_bf16(d.y), p.y0)
        with pytest.raises(lq.LqDeviceError, match="timed out"):
            lq.raise_on_device_error(ws, "forward")
    # the slab variant has no device-wide wait: it works on the same workspace as it is
    words[0] = 0
    lq.lora_segmented_forward(d.x, d.y, d.adapters, d.seg, h_out, ws, lq.LQ_VARIANT_SLAB)
    torch.cuda.synchronize()
    assert int(words[0].item()) == 0
    assert_close(synth.bf16_bits_to_f64(lq.bits_from_bf16(d.y)), ref.y, "y after the slab call")
    d.y.copy_(lq.bf16_from_bits(p.y0))
    # two launches do not use the barrier words: same workspace, error word cleared by the caller
    words[0] = 0
    lq.lora_segmented_forward(d.x, d.y, d.adapters, d.seg, h_out, ws, lq.LQ_VARIANT_SPLIT)
    torch.cuda.synchronize()
    assert int(words[0].item()) == 0
    assert_close(synth.bf16_bits_to_f64(lq.bits_from_bf16(d.y)), ref.y, "y after the two-launch call")
    # header zeroed: the single launch works again
    ws.zero_()
    d.y.copy_(lq.bf16_from_bits(p.y0))
    lq.lora_segmented_forward(d.x, d.y, d.adapters, d.seg, h_out, ws, lq.LQ_VARIANT_FUSED)
    torch.cuda.synchronize()
    assert int(words[0].item()) == 0
    assert_close(synth.bf16_bits_to_f64(lq.bits_from_bf16(d.y)), ref.y, "y after the header was zeroed")


def test_one_workspace_many_calls(oracle_mod):
    """One workspace reused by consecutive calls (two launches, one launch, slabs, two launches, one launch, slabs) on a batch
    with many more units than resident workgroups, so that the ticket counters are drawn from: every call must
    match the oracle, and the header's counters must be back at zero after every call."""
    p = synth.config4("up")
    ref = oracle_mod.forward(p.x, p.y0, p.A, p.B, p.ranks, p.scales, p.batch.token_adapter, p.batch.token_kind)
    d = DeviceProblem(p)
    d.build()
    ws = lq.workspace(lq.lora_forward_workspace_bytes(p.n_tokens, d.adapters.max_rank, p.d_in, p.d_out, lq.LQ_VARIANT_FUSED))
    y0 = lq.bf16_from_bits(p.y0)
    for variant in (lq.LQ_VARIANT_SPLIT, lq.LQ_VARIANT_FUSED, lq.LQ_VARIANT_SLAB, lq.LQ_VARIANT_SPLIT, lq.LQ_VARIANT_FUSED,
                    lq.LQ_VARIANT_SLAB):
        d.y.copy_(y0)
        h_out = torch.full((ref.segments.h_elems,), float("nan"), dtype=torch.float32, device="cuda")
        lq.lora_segmented_forward(d.x, d.y, d.adapters, d.seg, h_out, ws, variant)
        torch.cuda.synchronize()
        header = ws.view(torch.int32)[:1024].cpu().numpy()
        assert header[0] == 0
        assert not np.any(header[np.arange(1024) != 32]), "counters of the header must be back at zero"  # word 32 counts barriers
        assert_close(synth.bf16_bits_to_f64(lq.bits_from_bf16(d.y)), ref.y, "y")
        assert_close(h_out.cpu().numpy(), ref.h, "h_out")


def test_slab_variant_runs_beside_other_kernels(oracle_mod):
    """The slab variant has no device-wide wait, so it needs no compute unit to itself: here it runs while another
    stream keeps the device busy with matrix products (the paper's setting: base-model work of other requests on the
    same GPU), and gives the oracle's result; the error word stays clean."""
    p = synth.config3()
    ref = oracle_mod.forward(p.x, p.y0, p.A, p.B, p.ranks, p.scales, p.batch.token_adapter, p.batch.token_kind)
    d = DeviceProblem(p)
    d.build()
    ws = lq.workspace(lq.lora_forward_workspace_bytes(p.n_tokens, d.adapters.max_rank, p.d_in, p.d_out, lq.LQ_VARIANT_SLAB))
    h_out = torch.full((ref.segments.h_elems,), float("nan"), dtype=torch.float32, device="cuda")
    a = torch.randn(4096, 4096, device="cuda", dtype=torch.bfloat16)
    b = torch.randn(4096, 4096, device="cuda", dtype=torch.bfloat16)
    other = torch.cuda.Stream()            # default priority
    torch.cuda.synchronize()
    with torch.cuda.stream(other):
        for _ in range(40):                # a few milliseconds of work on the other stream
            c = a @ b
    for _ in range(3):                     # meanwhile, on this stream
        d.y.copy_(lq.bf16_from_bits(p.y0))
        lq.lora_segmented_forward(d.x, d.y, d.adapters, d.seg, h_out, ws, lq.LQ_VARIANT_SLAB)
    torch.cuda.synchronize()
    assert c.shape == (4096, 4096)
    lq.raise_on_device_error(ws, "slab beside other kernels")
    assert_close(synth.bf16_bits_to_f64(lq.bits_from_bf16(d.y)), ref.y, "y")
    assert_close(h_out.cpu().numpy(), ref.h, "h_out")
