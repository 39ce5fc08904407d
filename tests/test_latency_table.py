"""The per-shape latency table (paper, Sec. 5.3 / Fig. 6): the choice function on a
hand-made table (CPU), and a short real sweep through the C ABI (GPU)."""
import pytest

from paper_2002_10711_amd import latency


def test_choose_algorithm_picks_the_fastest():
    table = {
        latency.shape_key(3, 32, 32, "f32"): {"im2row": 5.0, "F2": 7.0, "F4": 6.0, "F6": 9.0},
        latency.shape_key(64, 64, 16, "int8"): {"im2row": 50.0, "F2": 14.0, "F4": 11.0, "F6": 30.0},
    }
    assert latency.choose_algorithm(table, 3, 32, 32, "f32") == ("im2row", 5.0)
    assert latency.choose_algorithm(table, 64, 64, 16, "int8") == ("F4", 11.0)
    with pytest.raises(KeyError):
        latency.choose_algorithm(table, 64, 64, 8, "int8")
    md = latency.to_markdown({k: dict(v, best=latency.choose_algorithm(table, *_parse(k))[0])
                              for k, v in table.items()}, 1)
    assert md.count("\n") == 3 and "| F4 |" in md


def _parse(key):
    dtype, rest = key.split(":")
    ch, size = rest.split("@")
    c, k = ch.split("->")
    return int(c), int(k), int(size), dtype


@pytest.mark.gpu
def test_short_sweep_on_gpu():
    table = latency.sweep(N=4, sizes=(16, 4), channels=((3, 32), (64, 64)), reps=20, warmup=10)
    assert len(table) == 8
    for key, row in table.items():
        assert set(latency.ALGORITHMS) <= set(row)
        assert all(0.5 < row[a] < 1e5 for a in latency.ALGORITHMS), (key, row)
        assert row["best"] == latency.choose_algorithm(table, *_parse(key))[0]
