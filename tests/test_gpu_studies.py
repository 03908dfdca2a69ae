"""The side studies run end to end on a shrunken workload (their numbers
are not checked here, only that they complete, validate and report sane fields)."""
import pytest

pytestmark = pytest.mark.gpu


def test_rearrangement_study_small():
    from paper_2408_02937_amd import studies
    print("[case] rearrangement study, scale 0.03, thresholds 500 / 2000", flush=True)
    out = studies.rearrangement_study(scale=0.03, thresholds=(500, 2000), iters=5)
    for row in out["rows"]:
        assert row["runs_after"] == 1 and row["runs_before"] >= 1
        assert row["hot_list_len"] > row["threshold"]
        assert row["share_of_online_vectors_on_hot_list"] == 1.0
        assert row["rearrange_cost_ms"] > 0


def test_hot_list_rearrangement_study_small():
    from paper_2408_02937_amd import studies
    print("[case] hot-list rearrangement study, scale 0.002, thresholds 500 / 2000", flush=True)
    out = studies.hot_list_rearrangement_study(scale=0.002, thresholds=(500, 2000), iters=5)
    assert out["runs_after_first_rearrangement"] == 1
    for row in out["rows"]:
        assert row["runs_after"] == 1 and row["runs_before"] > 1
        assert row["share_of_online_vectors_on_hot_list"] == 1.0
        assert row["rearrange_cost_ms"] > 0 and row["latency_ms"]["256"]["after_p50"] > 0


def test_block_size_sweep_small():
    from paper_2408_02937_amd import studies
    print("[case] block size sweep, scale 0.03, T_m 64 / 256", flush=True)
    out = studies.block_size_sweep(scale=0.03, sizes=(64, 256), iters=5)
    pads = [r["pad_bytes"] for r in out["rows"]]
    assert pads[1] > pads[0] > 0
    for r in out["rows"]:
        assert r["search"]["256"]["scan_ms"] > 0


def test_pq_study_small():
    from paper_2408_02937_amd import studies
    print("[case] product-quantiser study, scale 0.03, M 16", flush=True)
    out = studies.pq_study(scale=0.03, ms=(16,), iters=5)
    r = out["rows"][0]
    assert r["pool_bytes"] < r["flat_pool_bytes"]  # (the fixed part of the pool dominates at this scale)
    assert 0.0 < r["share_of_flat_topk_returned"] <= 1.0
    assert r["search"]["256"]["scan_ms"] > 0


def test_storage_study_small():
    from paper_2408_02937_amd import studies
    print("[case] storage study, scale 0.03", flush=True)
    out = studies.storage_study(scale=0.03, iters=5, batches=(1, 32))
    byte_set, unit_set = out["sets"]
    assert [r["storage"] for r in byte_set["rows"]] == ["f32", "f16", "u8"]
    assert all(r["share_of_f32_topk_returned"] == 1.0 for r in byte_set["rows"])   # byte values survive both
    sizes = [r["block_bytes"] for r in byte_set["rows"]]
    assert sizes[0] > sizes[1] > sizes[2]
    assert unit_set["rows"][1]["share_of_f32_topk_returned"] > 0.9
    for r in byte_set["rows"] + unit_set["rows"]:
        assert r["search"]["32"]["scan_ms"] > 0


def test_shape_study_small():
    from paper_2408_02937_amd import studies
    print("[case] shape study, scale 0.02", flush=True)
    out = studies.shape_study(scale=0.02, iters=5)
    assert [r["d"] for r in out["rows"]] == [96, 768, 256]
    for r in out["rows"]:
        for v in r["search"].values():
            assert v["scan_ms"] > 0 and v["p50_ms"] > 0


def test_mixed_load_study_small():
    from paper_2408_02937_amd import studies
    print("[case] mixed load study, scale 0.02, 2000 operations/s for 0.5 s", flush=True)
    out = studies.mixed_load_study(scale=0.02, rates=(2_000,), seconds=0.5)
    r = out["rows"][0]
    assert r["query_latency_ms"]["n"] + r["insert_latency_ms"]["n"] > 0
    assert r["query_latency_ms"]["p50"] > 0


def test_growth_study_small():
    from paper_2408_02937_amd import studies
    print("[case] growth study, scale 0.05, 1 s at 50,000 vectors/s, threshold 500", flush=True)
    out = studies.growth_study(scale=0.05, seconds=1.0, rate=50_000.0, threshold=500)
    assert out["vectors_inserted"] > 0 and out["search"]["during"]["requests"] > 0
    h = out["hot_lists"][0]
    assert h["vectors_after"] > h["vectors_before"]
    # the hot list was compacted on the way (which of its last blocks still stand alone depends on when the
    # device's report of the last exceeding batch reached the host)
    assert h["runs_after"] <= max(3, h["blocks_after"] // 4)
    assert out["pool"]["lists_exceeding_after"] == 0


def test_online_latency_study_small():
    from paper_2408_02937_amd import studies
    print("[case] online latency study, scale 0.03, 1000 queries/s, 0 and 5000 vectors/s, 0.3 s each", flush=True)
    out = studies.online_latency_study(scale=0.03, search_rates=(1000,), insert_rates=(0, 5000), seconds=0.3)
    quiet, busy = out["rows"]
    assert quiet["insert_requests"] == 0 and quiet["search_requests"] == 300
    assert busy["insert_requests"] > 0 and busy["insert_avg_ms"] > 0
    assert busy["latency_avg_ms"] == pytest.approx(busy["search_avg_ms"] + busy["insert_avg_ms"])
