"""Host-side checks of the dependent-layer executor's task lists (no GPU): every row block of every
stage is covered once, every workgroup's list is in phase order, and a model of the grid -- each
workgroup walking its list, a task starting only when the tasks that produce its input are done --
always drains, while a list that breaks the ordering rule is caught as stuck after a bounded number
of rounds instead of looping for ever."""
import numpy as np
import pytest

from paper_2602_06694_amd import binding as nq
from paper_2602_06694_amd import synth


def block_spec(block, n_blocks):
    """Shapes, levels and producer indices of n_blocks decoder blocks chained through q -> o -> gate -> down -> next q."""
    d_out, d_in, r, level, src = [], [], [], [], []
    for b in range(n_blocks):
        base = 7 * b
        for li, s in enumerate(block):
            d_out.append(s.d_out); d_in.append(s.d_in); r.append(s.r)
            level.append(4 * b + (0, 0, 0, 1, 2, 2, 3)[li])
            src.append({0: base - 1 if b else -1, 1: base - 1 if b else -1, 2: base - 1 if b else -1,
                        3: base + 0, 4: base + 3, 5: base + 3, 6: base + 4}[li])
    return d_out, d_in, r, level, src


def simulate(tasks, n_wg, src, max_rounds, planned=None):
    """Runs the task lists; returns the number of tasks left when no workgroup can advance (0 = drained).
    `planned`: the complete lists (a stage's input is there once ALL its planned tasks have run)."""
    lists = [[] for _ in range(n_wg)]
    for t in tasks:
        lists[t[0]].append(t)
    n_of = {}
    for t in (planned or tasks):
        n_of[(t[2], t[3])] = n_of.get((t[2], t[3]), 0) + 1
    done = {}
    pos = [0] * n_wg
    left = len(tasks)
    for _ in range(max_rounds):
        progressed = False
        for w in range(n_wg):
            if pos[w] >= len(lists[w]):
                continue
            _, _, layer, stage, _, _, _ = lists[w][pos[w]]
            need = (layer, 0) if stage == 1 else ((src[layer], 1) if src[layer] >= 0 else None)
            if need is None or done.get(need, 0) == n_of[need]:
                done[(layer, stage)] = done.get((layer, stage), 0) + 1
                pos[w] += 1
                left -= 1
                progressed = True
        if left == 0 or not progressed:
            break
    return left


@pytest.mark.parametrize("which,n_blocks,n_wg", [("7b", 3, 256), ("70b", 2, 256), ("70b", 1, 64), ("7b", 1, 7), ("7b", 2, 1)])
def test_task_lists_cover_everything_once_and_drain(which, n_blocks, n_wg):
    block = synth.llama2_7b_block() if which == "7b" else synth.llama2_70b_block()
    d_out, d_in, r, level, src = block_spec(block, n_blocks)
    tasks = nq.nq_exec_plan_tasks(d_out, d_in, r, level, n_wg).tolist()
    # coverage: each row block of each (layer, stage) exactly once; waves per row block a power of two <= 16
    for i in range(len(d_out)):
        for stage in (0, 1):
            rows = r[i] if stage == 0 else d_out[i]
            n_rb = (rows + 127) // 128
            seen = np.zeros(n_rb, dtype=int)
            for wg, phase, layer, st, rb0, n, W in tasks:
                if layer == i and st == stage:
                    assert phase == 2 * level[i] + stage and W in (1, 2, 4, 8, 16) and 0 <= wg < n_wg
                    seen[rb0:rb0 + n] += 1
            assert (seen == 1).all(), (i, stage)
    # every workgroup walks its tasks in phase order
    last = {}
    for wg, phase, *_ in tasks:
        assert phase >= last.get(wg, -1)
        last[wg] = phase
    assert simulate(tasks, n_wg, src, max_rounds=len(tasks) + 1) == 0


def test_model_reports_a_stuck_grid_after_bounded_rounds():
    """The model's waits are bounded like the kernel's: lists that break the phase order (one workgroup's
    list reversed), or a producer that never shows up, end with tasks left over, not in an endless loop."""
    d_out, d_in, r, level, src = block_spec(synth.llama2_7b_block(), 2)
    tasks = nq.nq_exec_plan_tasks(d_out, d_in, r, level, 4).tolist()
    wg0 = [t for t in tasks if t[0] == 0]
    others = [t for t in tasks if t[0] != 0]
    assert simulate(others + wg0[::-1], 4, src, max_rounds=10 * len(tasks)) > 0
    missing = [t for t in tasks if not (t[2] == 3 and t[3] == 0 and t[4] == 0)]       # a task of o's stage 1 never runs
    assert simulate(missing, 4, src, max_rounds=10 * len(tasks), planned=tasks) > 0


def test_planner_rejects_bad_arguments():
    with pytest.raises(nq.NQError):
        nq.nq_exec_plan_tasks([128], [128], [64], [0], 0)
    with pytest.raises(nq.NQError):
        nq.nq_exec_plan_tasks([128, 128], [128, 128], [64, 64], [1, 0], 8)      # levels out of order
    with pytest.raises(nq.NQError):
        nq.nq_exec_plan_tasks([0], [128], [64], [0], 8)
