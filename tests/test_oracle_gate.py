"""Pins of the oracle's throughput-aware speculation control (Sec. 5.4 of the paper, last paragraph: acceptance
rates are monitored; pre-profiling gives the largest batch at which speculation still pays at each acceptance
rate; above it speculation is switched off)."""
import numpy as np

import oracle


def new_gate(table, probe_every=0):
    g = np.zeros(32, np.int32)
    g[4] = probe_every
    g[8:25] = table
    return g


def test_table_for_an_affine_step_time_is_the_closed_form():
    # t(M) = c0 + c1 M: speculation pays iff (1 + a K)(c0 + c1 b) >= c0 + c1 b (1 + K)  <=>  b <= a c0 / (c1 (1 - a))
    c0, c1, K, b_max = 18.0, 0.011, 8.0, 4096
    rows = np.array([1, 64, 512, 4096, 40000], np.int32)
    ms = (c0 + c1 * rows).astype(np.float32)
    t = oracle.gate_table(ms, rows, K, b_max)
    for i in range(17):
        a = i / 16
        want = b_max if a == 1.0 else min(b_max, int(np.floor(a * c0 / (c1 * (1 - a)) + 1e-6)))
        assert abs(int(t[i]) - want) <= 1, (i, t[i], want)      # float32 profile points: off by one at most
    assert t[0] == 0 and t[16] == b_max and np.all(np.diff(t) >= 0)


def test_table_with_a_weight_streaming_plateau():
    # flat up to 300 rows (weights dominate), then linear: small batches gain even at low acceptance rates
    rows = np.array([1, 300, 3000], np.int32)
    ms = np.array([10.0, 10.0, 100.0], np.float32)
    t = oracle.gate_table(ms, rows, 4.0, 1000)
    assert t[1] >= 60 and t[1] < 300        # rate 1/16: all rows of b (1 + K) still on the plateau => b <= 60 pays
    assert np.all(np.diff(t) >= 0)


def test_monitor_converges_to_the_rate_and_the_gate_follows_the_table():
    table = np.array([0] * 8 + [100] * 9, np.int32)             # speculate iff the rate bucket is >= 8 (50 %) at live <= 100
    g = new_gate(table)
    dt = at = 0
    dec = []
    for step in range(60):
        dec.append(oracle.gate_step(g, 64, dt, at))
        if dec[-1]:
            dt += 400
            at += 300 if step < 30 else 100                      # 75 % accepted, later 25 %
    assert all(dec[:30]) and g[7] == 60
    assert dec[31] == 1 and not any(dec[36:])                    # the decayed rate falls below the bucket within a few steps
    # fixed point of X <- X - (X >> 3) + x lies in [8x, 8x + 7]
    g2 = new_gate(np.full(17, 10 ** 6, np.int32))
    dt = at = 0
    for _ in range(200):
        oracle.gate_step(g2, 1, dt, at)
        dt += 50
        at += 20
    assert 400 <= g2[0] <= 407 and 160 <= g2[1] <= 167


def test_batch_above_the_table_switches_off_and_probes_return():
    table = np.full(17, 32, np.int32)
    g = new_gate(table, probe_every=4)
    dt = at = 0
    dec = []
    for step in range(20):
        on = oracle.gate_step(g, 64, dt, at)                     # 64 live sequences > 32: off, except the probes
        dec.append(on)
        if on:
            dt += 100
            at += 10
    assert dec == [0, 0, 0, 0, 1] * 4                            # four steps off, then one probing step
    g = new_gate(table, probe_every=0)
    assert [oracle.gate_step(g, 64, 0, 0) for _ in range(10)] == [0] * 10   # never probes
    assert [oracle.gate_step(g, 32, 0, 0) for _ in range(3)] == [1] * 3     # a batch that fits speculates again


def test_counter_wraparound_is_harmless():
    g = new_gate(np.full(17, 10, np.int32))
    oracle.gate_step(g, 1, 2 ** 32 - 50, 2 ** 32 - 20)
    d0, a0 = int(g[0]), int(g[1])
    oracle.gate_step(g, 1, (2 ** 32 - 50 + 120) % 2 ** 32, (2 ** 32 - 20 + 60) % 2 ** 32)
    assert g[0] == d0 - (d0 >> 3) + 120 and g[1] == a0 - (a0 >> 3) + 60
