"""The tuner's selection logic and the tuning table it writes, without a GPU: a stub timer stands
for the measurement, the table goes through JSON into emb_bag_set_tuning_table, and the planner
(which needs no GPU) must follow it - and stop following it when a key is set explicitly."""
import json

import pytest

import paper_2410_22249_amd as emb
from paper_2410_22249_amd import autotune
from tuning_ctx import tuning


def _plan(row_bytes, L, T=26, B=8192):
    desc = emb.make_desc(T, B, row_bytes // 4, emb.EMB_F32, emb.EMB_SUM, int(T * B * L), 0, 1_000_000)
    return emb.emb_bag_plan_forward(desc)


@pytest.fixture(autouse=True)
def _clean_table():
    yield
    emb.emb_bag_set_tuning_table([])


def test_choose_keeps_the_automatic_setting_within_the_margin():
    auto = (100e-6, {})
    assert autotune.choose([auto, (99e-6, {"depth": 8})])[1] == {}          # 1 %: noise
    assert autotune.choose([auto, (90e-6, {"depth": 8})])[1] == {"depth": 8}
    assert autotune.choose([auto, (120e-6, {"depth": 8})])[1] == {}


def test_sweep_table_roundtrip_and_planner(tmp_path):
    # a made-up machine: depth 8 pays for 512-byte rows with long bags, two bags per wavefront for
    # 256-byte rows at pooling 16, the stream kernel wins for one-hot lookups whatever the row
    def timer(rb, L, s):
        t = 100e-6
        if L == 1:
            t *= 0.5 if s.get("stream", -1) != 0 else 1.0     # automatic already streams one-hot bags
        if rb == 512 and L >= 64 and s.get("depth") == 8 and s.get("stream") == 0 \
                and s.get("bags_per_wave") == 1:
            t *= 0.8
        if rb == 256 and L == 16 and s.get("bags_per_wave") == 2 and s.get("depth") == 4 \
                and s.get("stream") == 0:
            t *= 0.7
        return t
    lines = []
    per_shape, report = autotune.sweep_table([256, 512], [1, 16, 64], autotune.TABLE_GRID, 0, 0, 0,
                                             timer=timer, log=lines.append)
    assert per_shape[(512, 64)] == {"stream": 0, "depth": 8, "bags_per_wave": 1}
    assert per_shape[(256, 16)] == {"stream": 0, "depth": 4, "bags_per_wave": 2}
    assert per_shape[(256, 1)] == {} and per_shape[(512, 1)] == {} and per_shape[(512, 16)] == {}
    assert len(lines) == 6 and len(report) == 6
    entries = autotune.table_entries(per_shape, [256, 512], [1, 16, 64])
    path = tmp_path / "table.json"
    path.write_text(json.dumps({"entries": entries}))
    assert autotune.load_table(str(path)) == 6
    # the planner follows the table ...
    p = _plan(512, 80)
    assert (p.kernel, p.depth, p.bags_per_wave) == (emb.EMB_KERNEL_WAVE, 8, 1)
    p = _plan(256, 20)                       # pooling 20 falls in the band of the shape (256, 16)
    assert (p.kernel, p.depth, p.bags_per_wave) == (emb.EMB_KERNEL_WAVE, 4, 2)
    assert _plan(256, 1).kernel == emb.EMB_KERNEL_STREAM          # nothing pinned: automatic
    assert _plan(128, 20).bags_per_wave == 2                      # narrower rows: first covering entry
    assert _plan(1024, 80).depth == 8                             # wider rows than any entry: automatic
    # ... an explicit key wins over it ...
    with tuning(bags_per_wave=5, depth=2):
        p = _plan(256, 20)
        assert (p.depth, p.bags_per_wave) == (2, 5)
    # ... and clearing the table restores the automatic choice
    emb.emb_bag_set_tuning_table([])
    assert _plan(512, 80).depth == 8 and _plan(256, 20).bags_per_wave != 2


def test_table_argument_errors():
    good = {"max_row_bytes": 256, "max_avg_len": 10.0}
    for bad in ({"max_row_bytes": 8}, {"max_avg_len": -1.0}, {"depth": 3}, {"bags_per_wave": 33},
                {"stream": 2}, {"bags_per_group": 64}):
        with pytest.raises(emb.EmbBagError) as ex:
            emb.emb_bag_set_tuning_table([{**good, **bad}])
        assert ex.value.status == -9
    with pytest.raises(emb.EmbBagError) as ex:
        emb.emb_bag_set_tuning_table([good] * 65)
    assert ex.value.status == -7
    emb.emb_bag_set_tuning_table([good] * 64)


@pytest.mark.gpu
def test_a_two_by_two_grid_on_the_gpu_gives_identical_bits():
    """The tuner on a real GPU, small: every setting of a depth x bags-per-wavefront grid gives the
    same output bit for bit (tuning is speed only), the per-shape sweep runs and writes entries,
    and a forward call under the loaded table equals the others."""
    import torch
    from inputgen import gen
    state = autotune._setup_wl(gen.workload("small_f32_d128"), 2)
    wl, arena, toff, dev_batches, descs, out, batches, _ = state
    outs = []
    for depth in (4, 8):
        for bpw in (1, 2):
            autotune.apply_tuning({**autotune.NEUTRAL, "depth": depth, "bags_per_wave": bpw, "stream": 0})
            assert autotune._time(state, 2, 1) > 0
            out.fill_(float("nan"))
            emb.emb_bag_forward(descs[0], arena, toff, dev_batches[0][0], dev_batches[0][1], None, out)
            torch.cuda.synchronize()
            outs.append(out.clone())
    autotune.apply_tuning(autotune.NEUTRAL)
    assert all(torch.equal(outs[0], o) for o in outs[1:]) and bool(torch.isfinite(outs[0]).all())
    per_shape, report = autotune.sweep_table([512], [16], {"stream": [0], "depth": [4, 8],
                                                           "bags_per_wave": [1, 2]},
                                             lookups=200_000, steps=3, warmup=1, log=lambda _l: None)
    entries = autotune.table_entries(per_shape, [512], [16])
    assert len(entries) == 1 and len(report) == 1 and report[0]["best_us"] > 0
    assert autotune.load_table(entries) == 1
    out.fill_(float("nan"))
    emb.emb_bag_forward(descs[0], arena, toff, dev_batches[0][0], dev_batches[0][1], None, out)
    torch.cuda.synchronize()
    assert torch.equal(outs[0], out)
