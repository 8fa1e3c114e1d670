"""No GPU: the table of tuned configurations (Section 3.8: results are kept and reused) -- host logic of the library."""
import os

import pytest

import paper_2504_19442_amd as agg


def _entry(tile=2, order=1, wgs=256, tried=18, ms=0.7125):
    r = agg.TuneResult()
    r.tile_config, r.tile_order, r.producer_workgroups, r.configs_tried, r.best_ms = tile, order, wgs, tried, ms
    return r


@pytest.fixture(autouse=True)
def _empty_table():
    agg.agg_tune_table_clear()
    yield
    agg.agg_tune_table_clear()


def test_put_get_and_missing_entries():
    assert agg.agg_tune_table_size() == 0
    assert agg.agg_tune_table_get(8, 8192, 7168, 8192) is None
    agg.agg_tune_table_put(8, 8192, 7168, 8192, _entry())
    agg.agg_tune_table_put(8, 4096, 3584, 4096, _entry(tile=0, order=0, wgs=128, ms=0.09))
    agg.agg_tune_table_put(8, 8192, 7168, 8192, _entry(tile=0))          # same key: replaced, not added
    assert agg.agg_tune_table_size() == 2
    got = agg.agg_tune_table_get(8, 8192, 7168, 8192)
    assert (got.tile_config, got.tile_order, got.producer_workgroups, got.configs_tried) == (0, 1, 256, 18)
    assert abs(got.best_ms - 0.7125) < 1e-6
    assert agg.agg_tune_table_get(4, 8192, 7168, 8192) is None           # the world size is part of the key
    assert agg.agg_tune_table_get(8, 8192, 7168, 4096) is None


@pytest.mark.parametrize("bad", [dict(tile=8), dict(tile=-1), dict(order=2), dict(wgs=-1), dict(wgs=5000), dict(ms=-1.0)])
def test_put_rejects_values_out_of_range(bad):
    with pytest.raises(agg.AggError) as e:
        agg.agg_tune_table_put(8, 64, 64, 64, _entry(**bad))
    assert e.value.code == agg.ERR_INVALID_ARG
    with pytest.raises(agg.AggError):
        agg.agg_tune_table_put(0, 64, 64, 64, _entry())
    assert agg.agg_tune_table_size() == 0


def test_save_load_round_trip_and_merge(tmp_path):
    p = str(tmp_path / "tuned.txt")
    agg.agg_tune_table_put(8, 8192, 7168, 8192, _entry())
    agg.agg_tune_table_put(4, 1024, 512, 256, _entry(tile=1, order=0, wgs=0, tried=6, ms=0.031))
    agg.agg_tune_table_save(p)
    text = open(p).read().splitlines()
    assert text[0] == "agg-tune-table 1" and text[1].startswith("#")
    assert "4 1024 512 256 1 0 0 6 0.031" in text and "8 8192 7168 8192 2 1 256 18 0.7125" in text
    agg.agg_tune_table_clear()
    agg.agg_tune_table_put(8, 8192, 7168, 8192, _entry(tile=0))          # the file's entry wins over this one
    agg.agg_tune_table_put(2, 128, 128, 128, _entry(tile=1))             # and this one stays
    assert agg.agg_tune_table_load(p) == 2
    assert agg.agg_tune_table_size() == 3
    assert agg.agg_tune_table_get(8, 8192, 7168, 8192).tile_config == 2
    assert agg.agg_tune_table_get(2, 128, 128, 128).tile_config == 1
    got = agg.agg_tune_table_get(4, 1024, 512, 256)
    assert (got.tile_config, got.tile_order, got.producer_workgroups, got.configs_tried) == (1, 0, 0, 6)


@pytest.mark.parametrize("body", [
    "",                                                       # no header
    "some-other-file 1\n8 64 64 64 0 0 0 1 0.5\n",            # wrong header
    "agg-tune-table 2\n",                                     # another version
    "agg-tune-table 1\n8 64 64 64 0 0 0 1\n",                 # a field missing
    "agg-tune-table 1\n8 64 64 64 0 0 0 1 0.5 7\n",           # a field too many
    "agg-tune-table 1\n8 64 64 64 9 0 0 1 0.5\n",             # tile shape out of range
    "agg-tune-table 1\n8 64 64 64 0 0 0 1 nan\n",             # not a time
    "agg-tune-table 1\n8 64 64 x4 0 0 0 1 0.5\n",             # not a number
    "agg-tune-table 1\n8 64 64 64 0 0 0 1 0.5\n" + "9" * 400 + "\n",   # an overlong line
])
def test_malformed_files_leave_the_table_as_it_was(tmp_path, body):
    p = str(tmp_path / "bad.txt")
    open(p, "w").write(body)
    agg.agg_tune_table_put(8, 8192, 7168, 8192, _entry())
    with pytest.raises(agg.AggError) as e:
        agg.agg_tune_table_load(p)
    assert e.value.code == agg.ERR_INVALID_ARG
    assert agg.agg_tune_table_size() == 1 and agg.agg_tune_table_get(8, 64, 64, 64) is None


def test_comments_blank_lines_and_missing_files(tmp_path):
    p = str(tmp_path / "ok.txt")
    open(p, "w").write("# written by hand\n\nagg-tune-table 1\n  # indented comment\n8 64 64 64 1 1 32 3 0.25\r\n\n")
    assert agg.agg_tune_table_load(p) == 1
    assert agg.agg_tune_table_get(8, 64, 64, 64).producer_workgroups == 32
    with pytest.raises(agg.AggError) as e:
        agg.agg_tune_table_load(str(tmp_path / "absent.txt"))
    assert e.value.code == agg.ERR_IO
    with pytest.raises(agg.AggError) as e:
        agg.agg_tune_table_save(str(tmp_path / "no_such_dir" / "t.txt"))
    assert e.value.code == agg.ERR_IO
    assert agg.agg_strerror(agg.ERR_NOT_FOUND) == "no such entry"
