"""Host logic of the serving-trace generator (request stream + first-come-first-served steps).

The generator restates the workload of the paper's benchmark appendix (App. E.1, E.3); these
tests pin it to the stated laws and to a step-by-step simulation written out naively here.
"""
import numpy as np
import pytest

from paper_2605_14217_amd import workloads as wl


def test_request_lengths_follow_the_stated_law():
    r = wl.request_stream(20000, 8, "uniform", l_max=2048, seed=1)
    # -1 + 18 exp(0.8 Z): median 17, mean 18 exp(0.32) - 1 = 23.8
    assert abs(np.median(r.prompt_len) - 17) <= 1
    assert abs(r.prompt_len.mean() - (18 * np.exp(0.32) - 1)) < 0.6
    assert r.prompt_len.min() >= 1 and r.prompt_len.max() <= 2046
    assert r.output_len.min() >= 2
    assert np.all(r.prompt_len + r.output_len <= 2048)
    # prompt + output uniform on [prompt + 2, l_max]: mean of the total = (p + 2 + l_max) / 2
    total = r.prompt_len + r.output_len
    assert abs(total.mean() - (r.prompt_len.mean() + 2 + 2048) / 2) < 15
    # clipping at a small l_max
    s = wl.request_stream(2000, 8, "uniform", l_max=16, seed=2)
    assert s.prompt_len.max() == 14 and np.all(s.prompt_len + s.output_len <= 16)


def test_adapter_mixes():
    n, N = 4000, 16
    assert np.all(wl.request_stream(n, N, "identical").adapter == 0)
    u = wl.request_stream(n, N, "uniform").adapter
    assert u.min() == 0 and u.max() == N - 1
    assert np.bincount(u, minlength=N).min() > n / N * 0.7
    d = np.bincount(wl.request_stream(n + 5, N, "distinct").adapter, minlength=N)
    assert d.max() - d.min() <= 1
    z = np.bincount(wl.request_stream(n, N, "skewed").adapter, minlength=N)
    want = (1 / np.arange(1, N + 1)) / np.sum(1 / np.arange(1, N + 1)) * n      # Zipf, exponent 1
    assert np.all(np.abs(z - want) < 5 * np.sqrt(want) + 5)
    with pytest.raises(ValueError):
        wl.request_stream(4, 2, "round-robin")


def _naive_steps(prompt, output, adapter, batch):
    """One engine step at a time, no run compression: list of per-step (len, prefill_len, adapter) lists."""
    slots = [None] * batch
    nxt, steps = 0, []
    while True:
        for i in range(batch):
            if slots[i] is None and nxt < len(prompt):
                slots[i] = {"req": nxt, "made": 0}
                nxt += 1
        if all(s is None for s in slots):
            return steps
        step = []
        for s in slots:
            if s is None:
                continue
            if s["made"] == 0:
                step.append((int(prompt[s["req"]]), int(prompt[s["req"]]), int(adapter[s["req"]])))
            else:
                step.append((1, 0, int(adapter[s["req"]])))
            s["made"] += 1
        steps.append(step)
        for i, s in enumerate(slots):
            if s is not None and s["made"] >= output[s["req"]]:
                slots[i] = None


@pytest.mark.parametrize("batch,seed", [(1, 0), (3, 1), (8, 2), (32, 3)])
def test_fcfs_steps_match_a_step_by_step_simulation(batch, seed):
    req = wl.request_stream(60, 5, "uniform", l_max=48, seed=seed)
    want = _naive_steps(req.prompt_len, req.output_len, req.adapter, batch)
    got = []
    for tab, repeat in wl.fcfs_steps(req, batch):
        assert tab.S <= batch and repeat >= 1
        step = list(zip(tab.seg_len.tolist(), tab.seg_prefill_len.tolist(), tab.seg_adapter.tolist()))
        if repeat > 1:
            assert all(p == 0 for _, p, _ in step)          # only decode-only steps repeat
        got.extend([step] * repeat)
    assert got == want
    # conservation: every prompt row once, one decode row per output token after the first
    pre = sum(p for step in got for _, p, _ in step)
    dec = sum(l - p for step in got for l, p, _ in step)
    assert pre == int(req.prompt_len.sum())
    assert dec == int((req.output_len - 1).sum())
