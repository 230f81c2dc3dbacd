"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host-side
logic (shape validation, blob layout, arena sizing, KV slot bookkeeping, argument checks of a
dry-run instance) behaves as the header says.  No kernel runs here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import workloads
from paper_2412_17246_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", params=[False, True], ids=["bf16", "fp32dbg"])
def lib(request):
    return B.load_library(fp32_debug=request.param)


def test_every_declared_symbol_is_exported_and_bound(lib):
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(bz_[a-z0-9_]+)\s*\(", text))
    assert declared, "no declarations found"
    assert declared == set(B.SIGNATURES), declared ^ set(B.SIGNATURES)
    for name in declared:
        assert getattr(lib, name) is not None


def test_build_info_distinguishes_the_two_builds():
    assert B.load_library(False).bz_build_info() == 0
    assert B.load_library(True).bz_build_info() == B.BZ_BUILD_FP32_DEBUG


@pytest.mark.parametrize("name", list(workloads.CONFIGS))
def test_layout_and_sizes_match_the_parameter_count(lib, name):
    s = workloads.CONFIGS[name]
    cfg = B.make_config(s, max_seqs=4, max_seq_len=512, max_tokens=128, kv_tokens=1024)
    sz, lay = B.bz_sizes(), B.bz_layer_layout()
    assert lib.bz_query_sizes(C.byref(cfg), C.byref(sz)) == 0
    assert lib.bz_layer_layout_of(C.byref(cfg), C.byref(lay)) == 0
    assert sz.layer_bytes == 2 * s.params_per_layer == lay.total
    assert sz.layer_stride % 256 == 0 and sz.layer_stride >= sz.layer_bytes
    assert sz.weights_arena_bytes == sz.layer_stride * s.L
    act = 4 if lib.bz_build_info() & 1 else 2
    assert sz.act_elem_bytes == act
    assert sz.kv_arena_bytes == s.L * 2 * 1024 * s.Hkv * s.d * act
    shapes = workloads.tensor_shapes(s)
    off = 0
    for t in workloads.TENSOR_ORDER:
        assert getattr(lay, t) == off and off % 16 == 0
        off += 2 * int(np.prod(shapes[t]))
    assert off == lay.total


def test_layer_bytes_of_the_five_configured_shapes(lib):
    # bytes per layer of the five shapes, 2 * (H*d*(2*Hq + 2*Hkv) + 3*H*F + 2*H), worked out by hand from the
    # configurations' shape parameters (the paper prints no sizes)
    want = {"tiny": 1_582_080, "7b": 404_766_720, "8b_gqa": 436_224_000, "13b": 634_408_960, "70b": 1_711_308_800}
    for name, nbytes in want.items():
        cfg = B.make_config(workloads.CONFIGS[name], max_seqs=1, max_seq_len=16, max_tokens=16, kv_tokens=16)
        sz = B.bz_sizes()
        assert lib.bz_query_sizes(C.byref(cfg), C.byref(sz)) == 0
        assert sz.layer_bytes == nbytes


@pytest.mark.parametrize("field,value", [("n_layers", 0), ("hidden", 100), ("head_dim", 96), ("n_kv_heads", 3),
                                         ("ffn", 13), ("max_seqs", 0), ("kv_tokens", 0), ("rms_eps", 0.0),
                                         ("n_q_heads", 48)])
def test_bad_configs_are_rejected(lib, field, value):
    cfg = B.make_config(workloads.CONFIGS["tiny"], max_seqs=4, max_seq_len=512, max_tokens=128, kv_tokens=1024)
    if field == "n_q_heads":
        cfg.n_kv_heads = 3       # 48/3 = 16 query heads per kv head: unsupported group size
    setattr(cfg, field, value)
    sz = B.bz_sizes()
    assert lib.bz_query_sizes(C.byref(cfg), C.byref(sz)) == -1
    h = C.c_void_p()
    assert lib.bz_create(C.byref(cfg), C.byref(h)) == -1 and not h.value


def test_strerror(lib):
    assert lib.bz_strerror(0) == b"ok"
    assert lib.bz_strerror(-5) == b"layer not resident yet"
    assert lib.bz_strerror(-99) == b"unknown status"


@pytest.fixture()
def dry(lib):
    inst = B.Instance(workloads.CONFIGS["tiny"], max_seqs=4, max_seq_len=100, max_tokens=64, kv_tokens=256,
                      dry_run=True, fp32_debug=bool(lib.bz_build_info() & 1))
    yield inst
    inst.close()


def _status(fn, *a):
    try:
        fn(*a)
    except B.BzError as e:
        return e.name
    return "BZ_OK"


def test_kv_slot_bookkeeping(dry):
    assert dry.kv_free_tokens() == 256
    dry.kv_reserve(0, 90)                                        # rounded up to 96 positions
    dry.kv_reserve(1, 96)
    assert _status(dry.kv_reserve, 1, 10) == "BZ_EBUSY"
    assert _status(dry.kv_reserve, 2, 101) == "BZ_ECAPACITY"     # above max_seq_len
    assert _status(dry.kv_reserve, 2, 65) == "BZ_ECAPACITY"      # 64 positions left
    assert dry.kv_free_tokens() == 64
    dry.kv_release(0)
    assert dry.kv_free_tokens() == 96                            # two runs: 96 and 64, not adjacent
    dry.kv_reserve(2, 64)
    dry.kv_release(1)
    assert dry.kv_free_tokens() == 192                           # runs 0..96 and 96..192 merged
    dry.kv_release(2)
    assert dry.kv_free_tokens() == 256
    assert _status(dry.kv_release, 2) == "BZ_ESTATE"
    assert _status(dry.kv_reserve, 4, 10) == "BZ_EINVAL"


def test_kv_slot_allocator_against_a_model_on_random_sequences(lib):
    """Random reserve / release sequences on a dry-run instance against a few lines of Python that keep
    the set of occupied runs: first fit, requests rounded up to 32 positions, free runs merged."""
    rng = np.random.default_rng(11)
    for trial in range(20):
        n_slots = int(rng.integers(2, 24))
        total = int(rng.integers(4, 80)) * 32
        inst = B.Instance(workloads.CONFIGS["tiny"], max_seqs=n_slots, max_seq_len=total, max_tokens=8, kv_tokens=total,
                          dry_run=True, fp32_debug=bool(lib.bz_build_info() & 1))
        held = {}                                            # slot -> (offset, length)

        def free_runs():
            runs, at = [], 0
            for off, ln in sorted(held.values()):
                if off > at:
                    runs.append((at, off - at))
                at = off + ln
            if at < total:
                runs.append((at, total - at))
            return runs

        for step in range(200):
            slot = int(rng.integers(0, n_slots))
            if slot in held and rng.random() < 0.6:
                inst.kv_release(slot)
                del held[slot]
            else:
                want = int(rng.integers(1, total // 2 + 2))
                need = (want + 31) // 32 * 32
                got = _status(inst.kv_reserve, slot, want)
                if slot in held:
                    assert got == "BZ_EBUSY"
                else:
                    fit = next(((off, ln) for off, ln in free_runs() if ln >= need), None)
                    if want > total or fit is None:
                        assert got == "BZ_ECAPACITY", (trial, step, want, free_runs())
                    else:
                        assert got == "BZ_OK", (trial, step, want, free_runs())
                        held[slot] = (fit[0], need)
            assert inst.kv_free_tokens() == max([ln for _, ln in free_runs()], default=0)
        inst.close()


def test_frontier_and_argument_checks_without_a_gpu(dry):
    assert dry.frontier() == 0
    assert dry.layer_ready(0) is False
    assert _status(dry.wait_layer, 0) == "BZ_ENOTLOADED"
    assert _status(dry.wait_layer, 2) == "BZ_EINVAL"
    buf = np.zeros(dry.layer_bytes, dtype=np.uint8)
    lib, h = dry.lib, dry.handle
    assert lib.bz_load_layer(h, 0, buf.ctypes.data, buf.size - 1) == -1        # wrong size
    assert lib.bz_load_layer(h, 5, buf.ctypes.data, buf.size) == -1            # out of range
    assert lib.bz_load_layer(h, 0, None, buf.size) == -1
    assert lib.bz_load_layer(h, 0, buf.ctypes.data, buf.size) == -8            # dry run: validated, not enqueued
    assert lib.bz_readback_layer(h, 0, buf.ctypes.data) == -4
    assert lib.bz_export_boundary(h, 1, 65, 1, 0) == -7                        # T above max_tokens
    assert lib.bz_lend_second_copy_stream(h, None) == -1 and lib.bz_lend_second_copy_stream(None, 1) == -1
    assert lib.bz_lend_second_copy_stream(h, 1) == -8                          # dry run: no streams at all
    assert lib.bz_load_layer_from_peer(h, 0, h) == -1 and lib.bz_load_layer_from_peer(h, 0, None) == -1
    st = dry.stats()
    assert st["bytes_ingested"] == 0 and st["frontier"] == 0


def test_batch_descriptor_validation(lib):
    def make(q, s, k):
        q, s, k = (np.asarray(v, dtype=np.int32) for v in (q, s, k))
        d = B.bz_batch_desc(len(s), q.ctypes.data_as(C.POINTER(C.c_int32)), s.ctypes.data_as(C.POINTER(C.c_int32)),
                            k.ctypes.data_as(C.POINTER(C.c_int32)))
        h = C.c_void_p()
        return lib.bz_batch_create(C.byref(d), C.byref(h)), h
    assert make([1, 4], [0], [0])[0] == -1          # q_start[0] != 0
    assert make([0, 4, 2], [0, 1], [0, 0])[0] == -1  # decreasing offsets
    assert make([0, 2, 4], [1, 1], [0, 0])[0] == -1  # duplicate slot
    assert make([0, 2], [0], [-1])[0] == -1         # negative cache length
    assert make([0, 0], [0], [0])[0] == -1          # no tokens at all
    assert lib.bz_batch_create(None, C.byref(C.c_void_p())) == -1


def test_scheduler_decisions_match_the_oracle_in_virtual_time():
    """The C++ decision code, driven in virtual time, against the CPU oracle's simulation: integer
    configurations and finish times must agree exactly, for both policies."""
    from oracle import zigzag as Z
    cases = [(7, 7, 6.0, 1.0), (4, 3, 2.0, 0.0), (8, 10, 3.0, 5.0), (5, 6, 0.5, 2.0), (6, 4, 10.0, 0.0),
             (3, 8, 1.0, 1.0), (12, 5, 7.0, 30.0), (32, 12, 6.0, 1.0), (80, 6, 2.5, 0.0), (2, 2, 0.0, 0.0),
             # the source becomes free while the target is inside a layer
             (7, 5, 2.0, 1.5), (6, 6, 1.0, 0.25), (5, 4, 2.5, 3.75), (5, 1, 1e6, 0.5)]
    for L, n, load, free in cases:
        T, fin = B.zz_simulate(B.BZ_ZZ_ZIGZAG, L, n, load, free)
        want = Z.simulate_zigzag(L, n, load, free)
        assert T == want.T and fin == want.finish, (L, n, load, free)
        T, fin = B.zz_simulate(B.BZ_ZZ_BEST_EFFORT, L, n, load, free)
        want = Z.simulate_best_effort(L, n, load, free)
        assert T == want.T and fin == want.finish, (L, n, load, free)
    lib = B.load_library()
    assert lib.bz_zz_simulate(5, 3, 3, 1.0, 0.0, (C.c_int32 * 3)(), (C.c_double * 3)()) == -1     # unknown policy
    assert lib.bz_zz_create(None, None, 0, C.byref(C.c_void_p())) == -1


def test_scheduler_decisions_with_a_time_per_layer_and_request_match_the_oracle():
    """Section 5.4's retrofit: one layer of request r takes layer_time[r].  Times are sums and products of small
    dyadic numbers, so both sides compute them exactly and must agree bit for bit."""
    import random
    from oracle import zigzag as Z
    rnd = random.Random(5)
    for case in range(200):
        L, n = rnd.randint(1, 12), rnd.randint(1, 10)
        load = rnd.choice([0.0, 0.5, 1.0, 2.25, 6.0, 40.0])
        free = rnd.choice([0.0, 0.75, 3.0, 10.0, 100.0])
        w = [rnd.choice([0.25, 0.5, 1.0, 1.5, 3.0, 8.0]) for _ in range(n)]
        for policy, sim in ((B.BZ_ZZ_ZIGZAG, Z.simulate_zigzag), (B.BZ_ZZ_BEST_EFFORT, Z.simulate_best_effort)):
            T, fin = B.zz_simulate(policy, L, n, load, free, layer_time=w)
            want = sim(L, n, load, free, layer_time=w)
            assert T == want.T and fin == want.finish, (case, policy, L, n, load, free, w)
    # arbitrary floating-point load times, busy times and layer times, one-layer models included
    for case in range(400):
        L, n = rnd.randint(1, 40), rnd.randint(1, 12)
        load = rnd.choice([0.0, rnd.uniform(1e-3, 0.5), rnd.uniform(0.5, 20), rnd.uniform(20, 500)])
        free = rnd.choice([0.0, rnd.uniform(0, 5), rnd.uniform(5, 300)])
        w = [rnd.uniform(0.05, 5) for _ in range(n)] if rnd.random() < 0.6 else None
        for policy, sim in ((B.BZ_ZZ_ZIGZAG, Z.simulate_zigzag), (B.BZ_ZZ_BEST_EFFORT, Z.simulate_best_effort)):
            T, fin = B.zz_simulate(policy, L, n, load, free, layer_time=w)
            want = sim(L, n, load, free, layer_time=w)
            assert T == want.T and fin == want.finish, (case, policy, L, n, load, free, w)
    # load times whose multiples are not exact in binary: both sides count residency against the same products
    for load in (8.07, 0.1, 1.0 / 3.0, 7.3, 2.7, 1e-3, 123.456):
        for L, n, free in ((32, 6, 0.0), (7, 7, 1.0), (5, 9, 2.5)):
            for policy, sim in ((B.BZ_ZZ_ZIGZAG, Z.simulate_zigzag), (B.BZ_ZZ_BEST_EFFORT, Z.simulate_best_effort)):
                T, fin = B.zz_simulate(policy, L, n, load, free)
                want = sim(L, n, load, free)
                assert T == want.T and fin == want.finish, (policy, L, n, load, free)
    # the hand-worked timeline of the oracle's pins, through the C ABI as well
    assert B.zz_simulate(B.BZ_ZZ_ZIGZAG, 4, 2, 3.0, 2.0, layer_time=[1, 2]) == ([1, 2], [5.0, 9.0])
    assert B.zz_simulate(B.BZ_ZZ_BEST_EFFORT, 4, 2, 3.0, 2.0, layer_time=[1, 2]) == ([1, 1], [5.0, 11.0])
    # factors that are not positive, or not numbers, are refused
    for bad in ([1.0, 0.0], [1.0, -2.0], [float("nan"), 1.0], [float("inf"), 1.0]):
        with pytest.raises(B.BzError):
            B.zz_simulate(B.BZ_ZZ_ZIGZAG, 4, 2, 3.0, 2.0, layer_time=bad)


def _random_cluster(rng):
    n = int(rng.integers(2, 14))
    nodes = []
    for i in rng.permutation(40)[:n]:
        role = int(rng.choice([B.BZ_PLAN_SOURCE, B.BZ_PLAN_SPARE, B.BZ_PLAN_SPARE, B.BZ_PLAN_OTHER]))
        nodes.append((int(i), int(rng.choice([1, 2, 4, 8])), float(rng.choice([12.5e9, 25e9, 50e9])),
                      int(rng.integers(0, 4)), role, bool(rng.random() < 0.3)))
    return nodes


def test_scale_plan_matches_the_oracle_on_random_clusters():
    """The C++ planner against the CPU oracle: same chains, same hop bandwidths, same ready times
    (both evaluate the same float64 expressions), same interference flag and tails."""
    from oracle import multicast_plan as P
    rng = np.random.default_rng(5)
    checked = 0
    for _ in range(300):
        nodes = _random_cluster(rng)
        onodes = [P.Node(id=i, n_gpus=g, gpu_bw=bw, leaf=leaf, role=role, out_busy=busy)
                  for i, g, bw, leaf, role, busy in nodes]
        n_spare = sum(1 for n in onodes if n.role == P.SPARE)
        has_src = any(n.role == P.SOURCE for n in onodes)
        oversub = float(rng.choice([1.0, 2.0, 4.0]))
        L, layer = int(rng.integers(1, 40)), float(rng.choice([1.6e6, 4.05e8, 1.7e9]))
        for n_t in sorted({1, max(1, n_spare // 2), max(1, n_spare)}):
            if not has_src or n_t > n_spare:
                with pytest.raises(B.BzError) as e:
                    B.plan_generate(nodes, n_t, oversub, L, layer)
                assert e.value.name == "BZ_ECAPACITY"
                continue
            want = P.generate(onodes, n_t, oversub)
            got = B.plan_generate(nodes, n_t, oversub, L, layer)
            assert got["chains"] == want.chains
            assert got["hop_bw"] == want.hop_bw
            assert got["tails"] == want.tails and got["interferes"] == want.interferes
            assert got["ready"] == P.plan_ready_times(want, L, layer)
            checked += 1
    assert checked > 200


def test_scale_plan_argument_checks():
    ok = [(0, 1, 25e9, 0, B.BZ_PLAN_SOURCE, False), (1, 1, 25e9, 0, B.BZ_PLAN_SPARE, False)]
    assert B.plan_generate(ok, 1, 1.0, 4, 1e6)["chains"] == [[0, 1]]
    for bad_nodes, args in [
        (ok, (0, 1.0, 4, 1e6)),                                   # no target asked for
        (ok, (1, 0.5, 4, 1e6)),                                   # oversubscription below 1
        (ok, (1, 1.0, 0, 1e6)),                                   # no layers
        (ok, (1, 1.0, 4, 0.0)),                                   # empty layers
        ([ok[0], (0, 1, 25e9, 0, B.BZ_PLAN_SPARE, False)], (1, 1.0, 4, 1e6)),      # duplicate id
        ([ok[0], (1, 0, 25e9, 0, B.BZ_PLAN_SPARE, False)], (1, 1.0, 4, 1e6)),      # node without GPUs
        ([ok[0], (1, 1, 0.0, 0, B.BZ_PLAN_SPARE, False)], (1, 1.0, 4, 1e6)),       # no bandwidth
        ([ok[0], (1, 1, 25e9, 0, 7, False)], (1, 1.0, 4, 1e6)),                    # unknown role
    ]:
        with pytest.raises(B.BzError) as e:
            B.plan_generate(bad_nodes, *args)
        assert e.value.name == "BZ_EINVAL", (bad_nodes, args)


@pytest.mark.parametrize("libname", ["libblitzlayer.so", "libblitzlayer_fp32dbg.so"])
def test_headers_compile_as_c_and_the_library_serves_a_plain_c_program(tmp_path, libname):
    """include/*.h are C headers: a C99 program (tests/c_abi/dry_run.c) is compiled with gcc -pedantic, linked
    against the library with no Python in the process, and exercises the GPU-free calls."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2412_17246_amd")
    exe = str(tmp_path / "dry_run")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
           os.path.join(root, "tests", "c_abi", "dry_run.c"), "-o", exe, "-L", pkg, "-l:" + libname,
           "-Wl,-rpath," + pkg, "-Wl,-rpath,/opt/rocm/lib"]
    if libname.endswith("fp32dbg.so"):
        cmd.insert(1, "-DEXPECT_FP32_DEBUG")
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert run.returncode == 0 and "all checks passed" in run.stdout, run.stdout + run.stderr
