"""bench.py's overlap figures as functions of one call's trace: closed forms and bounds on
synthetic two-stream schedules (no GPU)."""
import numpy as np

import bench


def simulate(copy_ms, comp_ms, n_slots, rng=None):
    """Two in-order streams, layer l's compute waits for its copy, the copy of layer l waits for
    the compute of layer l - n_slots (slot reuse): the quantities sp_get_stats reports."""
    L = len(copy_ms)
    c_end, m_end, c_beg, m_beg = [0.0] * L, [0.0] * L, [0.0] * L, [0.0] * L
    for l in range(L):
        c_beg[l] = max(c_end[l - 1] if l else 0.0, m_end[l - n_slots] if l >= n_slots else 0.0)
        c_end[l] = c_beg[l] + copy_ms[l]
        m_beg[l] = max(m_end[l - 1] if l else 0.0, c_end[l])
        m_end[l] = m_beg[l] + comp_ms[l]
    hidden = sum(max(0.0, min(c_end[i], m_end[j]) - max(c_beg[i], m_beg[j])) for i in range(L) for j in range(L))
    wall = max(c_end[-1], m_end[-1]) - min(c_beg[0], m_beg[0])
    return sum(copy_ms), hidden, sum(comp_ms), wall


def test_serial_schedule_has_zero_overlap_efficiency():
    # one slot: copy, compute, copy, compute ...
    m = bench.overlap_metrics(*simulate([2.0] * 8, [1.0] * 8, 1))
    assert m["overlap_efficiency"] == 0.0 and m["copy_hidden_frac"] == 0.0
    assert abs(m["copy_stream_idle_frac"] - 1.0 / 3.0) < 1e-3


def test_link_bound_double_buffer():
    # copy 7 ms, compute 1 ms, two slots: compute hides entirely under the next copy
    cb, hid, mb, wall = simulate([7.0] * 32, [1.0] * 32, 2)
    m = bench.overlap_metrics(cb, hid, mb, wall)
    assert abs(wall - (32 * 7.0 + 1.0)) < 1e-9
    assert abs(m["overlap_efficiency"] - 31.0 / 32.0) < 1e-3
    assert abs(m["copy_hidden_frac"] - 31.0 / (32 * 7.0)) < 1e-3
    assert m["copy_hidden_frac"] <= m["copy_hidden_frac_bound"] == round(1.0 / 7.0, 4)
    assert m["copy_stream_idle_frac"] < 0.01


def test_bounds_hold_on_random_schedules():
    rng = np.random.default_rng(0)
    for _ in range(200):
        L = int(rng.integers(1, 40))
        m = bench.overlap_metrics(*simulate(list(rng.uniform(0.1, 5, L)), list(rng.uniform(0.1, 5, L)),
                                            int(rng.integers(1, 5))))
        assert 0.0 <= m["overlap_efficiency"] <= 1.0
        assert 0.0 <= m["copy_hidden_frac"] <= m["copy_hidden_frac_bound"] + 1e-4 <= 1.0001
        assert 0.0 <= m["copy_stream_idle_frac"] <= 1.0


def test_empty_trace_gives_no_figures():
    m = bench.overlap_metrics(0.0, 0.0, 0.0, 0.0)
    assert all(v is None for v in m.values())
