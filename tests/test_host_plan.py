"""CPU-only checks of the C-ABI library: it loads, exports what include/tc.h
declares, and its host planner (profile, Alg. 1-2, layout, placement) agrees
with the oracle bit for bit.  No kernel is launched here."""

import os
import re

import numpy as np
import pytest

import paper_2511_14124_amd as T
import workloads as W
from oracle import tc_oracle as o

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "tc.h")).read()
    names = set(re.findall(r"\b(tc_[a-z_]+)\s*\(", hdr))
    assert {"tc_profile_order", "tc_plan_pools", "tc_plan_schedule", "tc_migrate_step", "tc_cache_stats"} <= names
    L = T.load_library()
    for n in sorted(names):
        assert hasattr(L, n), n


def test_the_device_array_of_the_allocation_free_entry_point_is_visible_to_the_loader():
    # tc_pack_static asks the runtime for the address of a file-scope device array by the
    # name the host code registered.  The runtime finds it only if the GPU code object
    # exports that name; an array the compiler left with local binding (it does, for one
    # marked `used`) makes the runtime abort the process at the first call.
    import subprocess
    import tempfile
    tools = "/opt/rocm/llvm/bin"
    if not all(os.path.exists(os.path.join(tools, t)) for t in ("llvm-objcopy", "clang-offload-bundler", "llvm-readelf")):
        pytest.skip("LLVM binary tools not installed")
    obj = os.path.join(ROOT, "paper_2511_14124_amd", "csrc", "tc_kernels.o")
    if not os.path.exists(obj):
        pytest.skip("object file of the kernels not kept by this build")
    with tempfile.TemporaryDirectory() as d:
        fat, co = os.path.join(d, "fat.bin"), os.path.join(d, "k.co")
        subprocess.check_call([os.path.join(tools, "llvm-objcopy"), "--dump-section", ".hip_fatbin=" + fat, obj,
                               os.path.join(d, "copy.o")])
        subprocess.check_call([os.path.join(tools, "clang-offload-bundler"), "--type=o", "--unbundle",
                               "--targets=hipv4-amdgcn-amd-amdhsa--gfx950", "--input=" + fat, "--output=" + co])
        table = subprocess.check_output([os.path.join(tools, "llvm-readelf"), "--dyn-syms", "-W", co], text=True)
    rows = [ln.split() for ln in table.splitlines() if ln.strip().endswith("scratch")]
    assert rows, "the code object exports no symbol for the array"
    assert all(r[3] == "OBJECT" and r[4] == "GLOBAL" and int(r[2]) == (4 << 30) // 16384 * 4 for r in rows), rows


def _oracle_plan(wl):
    st, te, rw, _ = wl.events()
    p = o.profile(wl.tensor_bytes.tolist(), wl.tensor_group.tolist(), st, te, rw)
    plan = o.plan_pools(p, wl.hbm_bytes, wl.host_bytes, wl.align, wl.literal_alg2,
                        getattr(wl, "smallest_first", False))
    return p, plan, o.place(p, plan)


def _check_plan(wl):
    tc = T.TensorCache.from_workload(wl)
    p, plan, pl = _oracle_plan(wl)
    c = tc.classes
    assert c["bytes"].tolist() == p.class_bytes and c["group"].tolist() == p.class_group
    assert c["count"].tolist() == p.count and c["used"].tolist() == p.used
    assert c["step_max"].tolist() == p.step_max
    assert c["stride"].tolist() == plan.stride
    assert c["gpu_count"].tolist() == plan.gpu_count and c["cpu_count"].tolist() == plan.cpu_count
    assert c["hbm_off"].tolist() == plan.gpu_off and c["host_off"].tolist() == plan.cpu_off
    assert (tc.plan.hbm_total, tc.plan.host_total, tc.plan.file_total) == (plan.gpu_total, plan.cpu_total, pl.file_total)
    assert (tc.plan.n_rows, tc.plan.n_steps) == (p.n_rows, p.n_steps)
    q = tc.placement
    assert q["final_tier"].tolist() == pl.final and q["slot"].tolist() == pl.slot
    assert q["file_off"].tolist() == pl.file_off and q["cls"].tolist() == p.class_of
    assert q["first_use"].tolist() == p.first_use
    tc.close()


@pytest.mark.parametrize("index", range(5))
def test_plan_and_placement_match_the_oracle_on_the_five_configs(index):
    _check_plan(W.config(index))


@pytest.mark.parametrize("seed", range(25))
def test_plan_and_placement_match_the_oracle_on_random_traces(seed):
    wl = W.random_workload(seed, n_tensors=40, n_steps=50, literal=(seed % 3 == 0),
                           host_frac=(0.3 if seed % 2 else 1.5))
    if seed % 5 == 0:                       # a step that names a tensor twice is one row
        wl.profile[3] = wl.profile[3] + [wl.profile[3][0]]
    _check_plan(wl)


def test_worked_example_placements():
    for wl, gpu, cpu, nvme in ((W.example_cpu_gpu(), [0, 1, 2], [3, 4, 5], []),
                               (W.example_cpu_gpu_nvme(), [0, 1, 2], [3, 4, 5], [6]),
                               (W.example_cpu_gpu_nvme_two_sizes(), [0, 1, 2], [3, 4, 5], [6])):
        tc = T.TensorCache.from_workload(wl)
        f = tc.placement["final_tier"]
        assert [t for t in range(wl.n_tensors) if f[t] == T.GPU] == gpu
        assert [t for t in range(wl.n_tensors) if f[t] == T.CPU] == cpu
        assert [t for t in range(wl.n_tensors) if f[t] == T.NVME] == nvme


def test_error_codes_and_call_order():
    tc = T.TensorCache()
    with pytest.raises(T.TcError) as e:
        tc.plan_schedule()
    assert e.value.code == -2                                  # TC_E_STATE
    with pytest.raises(T.TcError) as e:
        tc.profile_order([512, 512], [0, 0], [1, 0], [0, 1], [1, 1])      # steps out of order
    assert e.value.code == -1
    with pytest.raises(T.TcError) as e:
        # a step index in the middle that is larger than the last one: the tables are sized by the last
        # event's step, so this must be refused before anything is written
        tc.profile_order([512, 512], [0, 0], [0, 900, 1], [0, 1, 0], [1, 1, 1])
    assert e.value.code == -1 and "ordered" in str(e.value)
    with pytest.raises(T.TcError) as e:
        tc.profile_order([512, 512], [0, 0], [0, 1 << 28], [0, 1], [1, 1])  # step index of TC_MAX_STEPS
    assert e.value.code == -1
    with pytest.raises(T.TcError) as e:
        tc.profile_order([512, 512], [0, 0], [0, 0xFFFFFFFF], [0, 1], [1, 1])
    assert e.value.code == -1
    with pytest.raises(T.TcError) as e:
        tc.profile_order([512, 512], [0, 0], [0, 1], [0, 7], [1, 1])      # unknown tensor
    assert e.value.code == -1
    with pytest.raises(T.TcError) as e:
        tc.profile_order([8, 512], [0, 0], [0, 1], [0, 1], [1, 1])        # tensor too small
    assert e.value.code == -1
    tc.profile_order([512, 512], [0, 0], [0, 1], [0, 1], [1, 1])
    tc.n_tensors = 2
    with pytest.raises(T.TcError) as e:
        tc.plan_pools(100, (0, 0))                               # working set does not fit
    assert e.value.code == -3                                   # TC_E_CAPACITY
    with pytest.raises(T.TcError) as e:
        tc.plan_pools(4096, (4096, 0), align=100)
    assert e.value.code == -1
    tc.plan_pools(4096, (4096, 0))
    with pytest.raises(T.TcError) as e:
        tc.migrate_step(0, T.PRE, [0], [1])                      # not bound yet
    assert e.value.code == -2
    tc.close()


@pytest.mark.parametrize("index", range(5))
def test_smallest_first_plan_matches_the_oracle_on_the_five_configs(index):
    wl = W.config(index)
    wl.smallest_first = True
    _check_plan(wl)


def test_smallest_first_plan_matches_the_oracle_on_random_traces():
    for seed in range(30):
        wl = W.random_workload(300 + seed, n_tensors=40, sizes=(512, 1024, 4096, 33000), hbm_frac=0.2,
                               literal=(seed % 5 == 0))
        wl.smallest_first = True
        _check_plan(wl)


def test_random_malformed_profiles_are_refused_or_planned_and_never_take_the_process_down():
    # what the planner is handed comes from a caller: whatever is wrong with it (steps out of order, a
    # step index far beyond the others, unknown tensors, sizes under 16 bytes, bad groups and flags, a
    # budget of nothing) must come back as an error code, and what is right must be planned
    rng = np.random.default_rng(20261128)
    outcomes = {"planned": 0, -1: 0, -3: 0}
    for case in range(400):
        n_t, n_s = int(rng.integers(1, 60)), int(rng.integers(1, 40))
        sizes = rng.choice([16, 17, 100, 512, 4096, 33000], size=n_t).astype(np.uint64)
        group = rng.integers(0, 2, size=n_t)
        step, tensor, rw = [], [], []
        for k in range(n_s):
            for _ in range(int(rng.integers(0, 5))):
                step.append(k), tensor.append(int(rng.integers(0, n_t))), rw.append(int(rng.integers(1, 4)))
        broken = int(rng.integers(0, 10))
        if step:
            i = int(rng.integers(0, len(step)))
            if broken == 0:
                step[i] = n_s + int(rng.integers(1, 1 << 20))       # larger than the last event's, in the middle
            elif broken == 1:
                tensor[i] = n_t + int(rng.integers(0, 3))
            elif broken == 2:
                rw[i] = int(rng.choice([0, 4, 255]))
            elif broken == 3:
                step[i] = 0xFFFFFFFF
        if broken == 4:
            sizes[int(rng.integers(0, n_t))] = int(rng.integers(0, 16))
        elif broken == 5:
            group[int(rng.integers(0, n_t))] = 2
        tc = T.TensorCache()
        try:
            tc.profile_order(sizes, group, step, tensor, rw)
            total = int(sizes.sum())
            tc.plan_pools(int(total * rng.choice([0.0, 0.1, 0.5, 2.0])), (int(total * rng.choice([0.0, 0.3, 2.0])),) * 2,
                          align=int(rng.choice([256, 16, 4096, 3, 8])), flags=int(rng.integers(0, 16)))
            tc.plan_schedule()
            outcomes["planned"] += 1
        except T.TcError as e:
            assert e.code in (-1, -3), (case, e)
            outcomes[e.code] += 1
        finally:
            tc.close()
    assert outcomes["planned"] > 50 and outcomes[-1] > 50 and outcomes[-3] > 10, outcomes


def test_the_bindings_records_have_the_layout_the_header_declares(tmp_path):
    # every struct the binding mirrors, field by field: a C program compiled against include/tc.h prints
    # sizeof and offsetof, which must be what numpy / ctypes lay out (a field added on one side only would
    # otherwise shift every figure behind it without an error); the constants the two sides share as well
    import ctypes
    import subprocess
    from paper_2511_14124_amd import binding as B
    records = {"tc_tensor_desc": B.TENSOR_DESC, "tc_event": B.EVENT, "tc_pool_class": B.POOL_CLASS,
               "tc_placement": B.PLACEMENT, "tc_op": B.OP, "tc_segment": B.SEGMENT,
               "tc_budget": B.Budget, "tc_pool_plan": B.PoolPlan, "tc_stats": B.Stats, "tc_timing": B.Timing}
    consts = {"TC_GPU": B.GPU, "TC_CPU": B.CPU, "TC_NVME": B.NVME, "TC_PRE": B.PRE, "TC_POST": B.POST,
              "TC_END": B.END, "TC_END_CPU": B.END_CPU, "TC_NONE": B.NONE, "TC_MAX_STEP_TENSORS": B.MAX_STEP_TENSORS,
              "TC_ALLOC_WRITE_ONLY": B.ALLOC_WRITE_ONLY, "TC_BIND_NULL_MOVER": B.BIND_NULL_MOVER,
              "TC_BIND_FILE_DIRECT": B.BIND_FILE_DIRECT, "TC_BIND_HOST_TIER": B.BIND_HOST_TIER}

    def fields(rec):
        if isinstance(rec, np.dtype):
            return rec.itemsize, [(n, rec.fields[n][1]) for n in rec.names]
        return ctypes.sizeof(rec), [(n, getattr(rec, n).offset) for n, _ in rec._fields_]

    lines = ['#include <stddef.h>', '#include <stdio.h>', '#include "tc.h"', 'int main(void) {']
    for name, rec in records.items():
        lines.append(f'  printf("{name} %zu", sizeof({name}));')
        for f, _ in fields(rec)[1]:
            lines.append(f'  printf(" %zu", offsetof({name}, {f}));')
        lines.append('  printf("\\n");')
    for name in consts:
        lines.append(f'  printf("{name} %llu\\n", (unsigned long long)({name}));')
    lines.append('  return 0; }')
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout.bin"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    out = subprocess.check_output([str(exe)], text=True).split("\n")
    got = {ln.split()[0]: [int(x) for x in ln.split()[1:]] for ln in out if ln}
    for name, rec in records.items():
        size, fs = fields(rec)
        assert got[name] == [size] + [off for _, off in fs], name
    for name, value in consts.items():
        assert got[name] == [value], name


def test_every_bound_function_takes_as_many_arguments_as_the_header_declares():
    # ctypes checks nothing against the header: an argument left out of a prototype in the binding would
    # shift the ones behind it silently.  Every declaration of include/tc.h, comments stripped, against the
    # argument list the binding registered for that symbol.
    import ctypes
    hdr = re.sub(r"/\*.*?\*/", " ", open(os.path.join(ROOT, "include", "tc.h")).read(), flags=re.S)
    decls = re.findall(r"\b(int|const char \*|uint64_t)\s*(tc_[a-z_0-9]+)\s*\(([^;{]*?)\)\s*;", hdr)
    assert len(decls) > 40
    L = T.load_library()
    checked = 0
    for ret, name, params in decls:
        fn = getattr(L, name)
        n = 0 if params.strip() in ("", "void") else params.count(",") + 1
        if fn.argtypes is None:
            continue                                       # (a symbol the binding does not call)
        assert len(fn.argtypes) == n, (name, params)
        assert (fn.restype is ctypes.c_char_p) == ret.startswith("const char"), name
        checked += 1
    assert checked > 40
