"""Host logic of bench.py: the run lengths of every leg must fit the handle that is sized from them."""
import itertools

import bench


def test_run_lengths_cover_every_leg():
    for max_prompt, settle, warmup, steps, prof, n_cal in itertools.product(
            (1, 16, 512, 1024), (0, 32), (0, 5, 16), (1, 20, 64, 1024), (1, 64, 200), (64, 96)):
        for lead in (0, 64):
            free = bench.run_lengths(max_prompt, settle, warmup, steps, prof, n_cal, lead)
            # a free-running row may be `lead` tokens ahead of the slowest when the timed region ends
            assert free["timed_new"] >= settle + warmup + steps + lead
            assert max_prompt + free["timed_new"] <= free["max_seq"] and max_prompt + free["profile_new"] <= free["max_seq"]
        ln = bench.run_lengths(max_prompt, settle, warmup, steps, prof, n_cal)
        # no leg (timed run, per-kernel timing run, calibration runs) may ask for more tokens than the handle holds
        for leg_new in (ln["timed_new"], ln["profile_new"], ln["cal_new"]):
            assert max_prompt + leg_new <= ln["max_seq"], (max_prompt, settle, warmup, steps, prof, n_cal)
        assert ln["timed_new"] == settle + warmup + steps
        assert 1 <= ln["profile_steps"] <= max(steps, 1) and ln["profile_steps"] <= max(prof, 1)
        assert ln["profile_new"] == settle + warmup + ln["profile_steps"]


def test_fewer_steps_than_profile_steps():
    """The case that used to overflow: --steps 20 --warmup 5 with the default 64 profile steps."""
    ln = bench.run_lengths(512, 0, 5, 20, 64, 96)
    assert ln["profile_steps"] == 20 and ln["profile_new"] == 25
    assert ln["max_seq"] >= 512 + 96


def test_workload_table_is_consistent():
    assert bench.DEFAULT_WORKLOAD in bench.WORKLOADS
    for name, (pair, batch, plo, phi, steps, rule, d_min) in bench.WORKLOADS.items():
        assert batch >= 1 and 0 <= plo <= phi and steps >= 1 and d_min >= 1, name
        if rule is not None:
            assert rule[0] in ("share", "percentile"), name
            assert (0 < rule[1] < 1) if rule[0] == "share" else (0 < rule[1] < 100), name


def test_host_cpu_reads_cpuinfo():
    name, cores = bench.host_cpu()
    assert name is None or isinstance(name, str)
    assert cores is None or cores >= 1


def test_host_memory_reading():
    avail = bench.host_mem_available()
    assert avail is None or avail > 1e8
