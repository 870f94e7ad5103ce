"""Pins of the counter-based schedule generator's reference."""
import numpy as np

from oracle import schedule_gen as sg


def test_rates_ranges_and_independence():
    n, eR, eC, d_max = 4096, 5000, 3000, 6
    p_act = np.linspace(0.05, 1.0, n).astype(np.float32)
    acc = np.zeros(n)
    delays = np.zeros(d_max + 1)
    drops = 0
    R = 60
    prev = None
    for r in range(R):
        q = sg.generate_round(11, r, n, eR, eC, p_act, d_max, 0.2)
        acc += q["active"]
        delays += np.bincount(q["delay_R"], minlength=d_max + 1) + np.bincount(q["delay_C"], minlength=d_max + 1)
        drops += q["drop_R"].sum() + q["drop_C"].sum()
        assert q["delay_R"].min() >= 0 and q["delay_C"].max() <= d_max
        if prev is not None:
            assert abs(np.corrcoef(prev["delay_R"], q["delay_R"])[0, 1]) < 0.06
        prev = q
    assert np.abs(acc / R - p_act).max() < 0.25 and abs((acc / R - p_act).mean()) < 0.01
    assert acc[-1] == R                      # probability one is always active
    np.testing.assert_allclose(delays / delays.sum(), 1 / (d_max + 1), atol=0.004)
    assert abs(drops / (R * (eR + eC)) - 0.2) < 0.004
    a = sg.generate_round(11, 7, n, eR, eC, p_act, d_max, 0.2)
    b = sg.generate_round(11, 7, n, eR, eC, p_act, d_max, 0.2)
    c = sg.generate_round(12, 7, n, eR, eC, p_act, d_max, 0.2)
    assert all(np.array_equal(a[k], b[k]) for k in a if a[k] is not None)
    assert not np.array_equal(a["delay_R"], c["delay_R"])
    # different streams are not copies of each other
    assert not np.array_equal(a["delay_R"][:eC], a["delay_C"][:eC])


def test_sampled_rows_are_a_permutation_prefix():
    for samples, batch in ((2048, 64), (100, 100), (37, 12), (1, 1), (2, 2), (513, 200)):
        firsts = []
        for r in range(40):
            rows = sg.sample_rows(3, r, 5, batch, samples)
            assert rows.min() >= 0 and rows.max() < samples and len(set(rows.tolist())) == batch
            firsts.append(int(rows[0]))
        if samples >= 37:
            assert len(set(firsts)) > 20      # varies with the round
    full = sg.sample_rows(9, 0, 0, 2048, 2048)
    assert sorted(full.tolist()) == list(range(2048))
    # spread: mean of the first 256 of 2048 close to the middle
    assert abs(full[:256].mean() - 1023.5) < 120
    assert not np.array_equal(sg.sample_rows(9, 0, 0, 32, 2048), sg.sample_rows(9, 0, 1, 32, 2048))


def test_event_selection_is_one_hot_with_the_stated_frequencies():
    """Algorithm 2 activates exactly one agent per global iteration; the empirical
    frequencies follow the weights; zero-weight agents are never drawn."""
    n, K = 12, 6000
    w = np.array([0, 1, 1, 4, 0.5, 0, 2, 1, 1, 1, 0.25, 0], dtype=np.float32)
    counts = np.zeros(n)
    for k in range(K):
        q = sg.generate_event(5, k, n, 20, 20, w, 3, 0.1)
        assert q["active"].sum() == 1
        counts += q["active"]
    assert counts[w == 0].sum() == 0
    np.testing.assert_allclose(counts / K, w / w.sum(), atol=4 * np.sqrt(0.25 / K))
    uni = np.zeros(5)
    for k in range(3000):
        uni += sg.generate_event(6, k, 5, 4, 4, None, 0, 0.0)["active"]
    np.testing.assert_allclose(uni / 3000, 0.2, atol=0.03)
    # thresholds: monotone, closed at the top; delays and drops are those of the round generator
    cdf = sg.selection_thresholds(w, n)
    assert np.all(np.diff(cdf.astype(np.int64)) >= 0) and int(cdf[-1]) == 0xFFFFFFFF
    a, b = sg.generate_event(5, 9, n, 20, 20, w, 3, 0.1), sg.generate_round(5, 9, n, 20, 20, 0.5, 3, 0.1)
    assert all(np.array_equal(a[k], b[k]) for k in ("delay_R", "delay_C", "drop_R", "drop_C"))
