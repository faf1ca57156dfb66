"""The shipped tuning table against the timings it was built from (paper Sec. IV-E: the table
holds, per collective, scale and message size, the choice with the minimum end-to-end time).
profiles/tuning_times.txt, written by the tuning suite in the same run as the table, records every
variant's time behind every row; each row of the table must be the least time among them, ties
(within the suite's stated window) going to the variant listed first."""
import os

from paper_2303_08374_amd import tune

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TABLE = os.path.join(ROOT, "paper_2303_08374_amd", "tuning", "mi355x.tbl")
TIMES = os.path.join(ROOT, "profiles", "tuning_times.txt")


def _table_rows():
    rows = {}
    with open(TABLE) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            op, dt, P, nbytes, variant = line.split()
            rows[(op, dt, int(P), int(nbytes))] = variant
    return rows


def test_tie_window():
    assert tune.tie_window_us(6.0) == 0.5                    # launch-bound: half a microsecond
    assert abs(tune.tie_window_us(60.0) - 1.2) < 1e-9        # 2 % below 100 us
    assert abs(tune.tie_window_us(1000.0) - 5.0) < 1e-9      # 0.5 % above
    assert tune.pick({"v1": 6.2, "v2": 6.0, "v4": 7.1}) == "v1"
    assert tune.pick({"v1": 6.6, "v2": 6.0, "v4": 7.1}) == "v2"
    assert tune.pick({"v1": 1000.0, "v2": 990.0, "v4": 900.0}) == "v4"
    assert tune.tie_window_us(4.0, graph_timed=True) == 0.1  # replayed from a graph: a tenth of a microsecond
    assert tune.pick({"v1": 4.8, "v2": 4.5, "v4": 4.45}, graph_timed=True) == "v2"
    assert tune.pick({"v1": 4.8, "v2": 4.5, "v4": 4.45}) == "v1"


def test_every_table_row_is_the_least_time_of_its_recorded_timings():
    table = _table_rows()
    times = tune.read_times(TIMES)
    assert len(times) == len(table) >= 4 * 2 * 3 * 17           # collectives x dtypes x scales x sizes, plus the workload ops
    for op, dt, P, nbytes, chosen, us, how in times:
        assert how in ("batch", "graph")
        graph_timed = how == "graph"
        key = (op, dt, P, nbytes)
        assert key in table, f"no table row for {key}"
        assert table[key] == chosen, f"{key}: table says {table[key]}, the timing record {chosen}"
        assert chosen in us
        best = tune.pick(us, graph_timed)
        assert best == chosen, f"{key}: {chosen} ({us[chosen]} us) is not the pick of {us}"
        floor = min(us.values())
        assert us[chosen] <= floor + tune.tie_window_us(floor, graph_timed)
