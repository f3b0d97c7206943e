"""Step-by-step invariants of a replay, checked on the oracle's state.

Capacity never exceeded, owner tables and tensor->slot maps mutual inverses,
every tensor in exactly one tier, every served access resident between the
pre- and the post-hook, hits + misses = accesses.
"""

from oracle import tc_oracle as o


def check_state(r, step, access, phase):
    p, plan = r.p, r.plan
    n_c = len(p.count)
    seen_gpu, seen_cpu = set(), set()
    for s in range(n_c):
        assert len(r.gpu_owner[s]) == plan.gpu_count[s]
        assert len(r.cpu_owner[s]) == plan.cpu_count[s]
        for k, t in enumerate(r.gpu_owner[s]):
            if t != o.NONE:
                assert r.cur[t] == o.GPU and r.gslot[t] == k and p.class_of[t] == s
                assert t not in seen_gpu
                seen_gpu.add(t)
        for k, t in enumerate(r.cpu_owner[s]):
            if t != o.NONE:
                assert r.cur[t] == o.CPU and r.cslot[t] == k and p.class_of[t] == s
                assert t not in seen_cpu
                seen_cpu.add(t)
            else:
                assert not r.designated[s][k]
    for t in range(p.n_tensors):
        if r.cur[t] == o.GPU:
            assert t in seen_gpu and r.cslot[t] == o.NONE
        elif r.cur[t] == o.CPU:
            assert t in seen_cpu and r.gslot[t] == o.NONE
        else:
            assert r.cur[t] == o.NVME and r.gslot[t] == o.NONE and r.cslot[t] == o.NONE
    assert sum(plan.gpu_count[s] * plan.stride[s] for s in range(n_c)) == plan.gpu_total
    if phase == o.PRE:
        res = r.resident_at_pre[-1]
        for (t, _a), where in zip(access, res):
            if where is not None:
                assert r.cur[t] == o.GPU and where == (p.class_of[t], r.gslot[t])
    if phase == o.END:
        for t in range(p.n_tensors):
            if r.fails == 0:
                assert r.cur[t] == r.pl.final[t], (t, r.cur[t], r.pl.final[t])
        assert r.cursor == 0
    assert r.hits + r.misses == sum(h + m for (_i, _k, h, m) in r.step_hits)
