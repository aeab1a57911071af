"""CPU-only tests of libferret's host side: the library loads and exports the whole C ABI,
the bucket planner's layout, the ring bookkeeping, and every argument error that is detected
before a HIP call.  No kernel is launched here."""
import os
import re

import pytest

from oracle import ferret_oracle as O
from paper_2503_12053_amd import binding as B
from paper_2503_12053_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2503_12053_amd import build
    build.build(verbose=False)          # no-op when the library is newer than its sources
    return B.load()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "ferret.h")).read() + \
        open(os.path.join(ROOT, "include", "ferret_planner.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ferret_[a-z0-9_]+)\s*\(", header))
    assert {"ferret_plan_buckets", "ferret_push_version", "ferret_compensate_step"} <= declared
    assert declared == set(B.SIGNATURES), declared ^ set(B.SIGNATURES)
    for name in declared:
        assert hasattr(lib, name), name
    assert b"gfx950" in lib.ferret_version()


def _plan(sizes_per_stage, tau, K=-1, R=None, prec=B.FERRET_F32, chunk=0, tuning=None):
    tensors = [(n, j) for j, sizes in enumerate(sizes_per_stage) for n in sizes]
    R = max(tau) + 1 if R is None else R
    return B.ferret_plan_buckets(tensors, len(sizes_per_stage), tau, K, R, prec, chunk, tuning), tensors


def test_library_reports_the_hash_of_the_sources_in_the_tree(lib):
    """ferret_version() ends with the hash of the code the library was built from; it must be the hash of the sources
    in this tree (a stale library fails here), and comments or white space do not change it."""
    from paper_2503_12053_amd import build
    assert lib.ferret_version().decode().split()[-1] == build.source_hash()
    code = 'int a = 1; const char *s = "// kept /* kept */"; char c = \'"\';'
    commented = 'int a = 1;   // the stage\'s "count"\n/* more\n "text" */ const char *s = "// kept /* kept */";\tchar c = \'"\';'
    assert build._code_only(commented) == build._code_only(code) == code


def test_layout_alignment_and_disjointness(lib):
    sizes = [[1, 3, 1001, 64], [7], [4096, 5]]
    plan, tensors = _plan(sizes, [2, 1, 0], R=3)
    assert plan.n_stages == 3 and plan.n_tensors == 7
    assert plan.total_params == sum(n for n, _ in tensors)
    # tensor offsets: aligned, in order, non-overlapping inside the stage
    i = 0
    for j, ss in enumerate(sizes):
        end = 0
        for n in ss:
            off = plan.tensor_offset(i)
            assert off % B.FERRET_ALIGN_ELEMS == 0 and off >= end
            end = off + n
            i += 1
        assert plan.stage_params(j) == sum(ss)
        assert plan.stage_numel(j) >= end and plan.stage_numel(j) % B.FERRET_ALIGN_ELEMS == 0
        assert plan.stage_numel(j) - end < B.FERRET_ALIGN_ELEMS
    # flat and ring regions: aligned to 16 bytes at least, disjoint, inside the totals
    flat, ring = [], []
    for j in range(3):
        fo, n = plan.stage_flat_offset(j), plan.stage_numel(j)
        assert fo % 4 == 0
        flat.append((fo, fo + n))
        stride, R = plan.stage_slot_stride(j), plan.stage_ring_depth(j)
        assert stride >= n and stride % 4 == 0 and R == 3
        for s in range(R):
            ring.append((plan.slot_offset(j, s), plan.slot_offset(j, s) + n))
    for regions, total in ((flat, plan.flat_elems), (ring, plan.ring_elems)):
        regions.sort()
        assert regions[0][0] >= 0 and regions[-1][1] <= total
        for a, b in zip(regions, regions[1:]):
            assert a[1] <= b[0]
    assert plan.ring_bytes == plan.ring_elems * 4 and plan.grad_bytes == plan.flat_elems * 4
    assert plan.master_bytes == plan.flat_elems * 4
    assert plan.workspace_bytes >= plan.n_chunks * 20


def test_chunks_never_cross_stage_boundaries(lib):
    plan, _ = _plan([[5000], [100], [3000, 3000]], [2, 1, 0], R=3, chunk=1024)
    per_stage = [-(-plan.stage_numel(j) // 1024) for j in range(3)]
    assert plan.chunk_elems == 1024 and plan.n_chunks == sum(per_stage)
    assert per_stage == [5, 1, 6]


def test_bf16_plan_sizes(lib):
    plan, _ = _plan([[100], [200]], [1, 0], R=2, prec=B.FERRET_BF16_MASTER_F32)
    assert plan.precision == B.FERRET_BF16_MASTER_F32
    assert plan.ring_bytes == plan.ring_elems * 2 and plan.grad_bytes == plan.flat_elems * 2
    assert plan.master_bytes == plan.flat_elems * 4
    assert [plan.stage_chunk_elems(j) for j in range(2)] == [2048, 2048] and plan.chunk_elems == 2048     # a small plan
    # with a byte target: K' = 1 has 2*(2+2)+8 = 16 bytes per element in flight, K' = 0 has 6+8 = 14
    sized, _ = _plan([[100], [200]], [1, 0], R=2, prec=B.FERRET_BF16_MASTER_F32, tuning=dict(chunk_bytes=48 * 1024))
    assert [sized.stage_chunk_elems(j) for j in range(2)] == [3072, 3072] and sized.chunk_elems == 3072


def test_default_chunks_move_equal_bytes_per_workgroup(lib):
    """For plans that stream, each stage's chunk is the multiple of 1024 elements nearest to 48 KiB / (bytes per
    element in flight), so a workgroup moves about the same bytes whatever its stage's K' (hand-computed for the
    ViT-B-sized workload and for Alg. 1's literal iteration count); plans that fit the memory-side cache keep 2048."""
    for idx in (1, 2, 3):
        small = B.plan_for_workload(W.make_workload(idx))
        assert {small.stage_chunk_elems(j) for j in range(small.n_stages)} == {2048}
    w = W.make_workload(4)
    plan = B.plan_for_workload(w)                     # K' = 3,3,3,3,3,2,1,0: 24,24,24,24,24,20,16,12 bytes per element
    assert [plan.stage_chunk_elems(j) for j in range(8)] == [2048] * 6 + [3072, 4096]
    assert [plan.stage_n_chunks(j) for j in range(8)] == [-(-plan.stage_numel(j) // plan.stage_chunk_elems(j)) for j in range(8)]
    assert plan.n_chunks == sum(plan.stage_n_chunks(j) for j in range(8))
    assert plan.workspace_bytes >= plan.n_chunks * 20
    full = B.plan_for_workload(w, n_iters=B.FERRET_ITERS_FULL)    # K' = 7..0: 40,36,32,28,24,20,16,12
    assert [full.stage_chunk_elems(j) for j in range(8)] == [1024, 1024, 2048, 2048, 2048, 2048, 3072, 4096]
    none = B.plan_for_workload(w, n_iters=0)          # no iterations: V[0] is still read for the weight gap (16 bytes)
    assert [none.stage_chunk_elems(j) for j in range(8)] == [3072] * 7 + [4096]
    deep = B.plan_for_workload(W.make_workload(5), n_iters=B.FERRET_ITERS_FULL)
    # bf16, K' = 15..0: beyond K' = 8 the kernel streams 8 versions at a time: 2*(8+2)+8 = 28 bytes in flight
    assert [deep.stage_chunk_elems(j) for j in range(7)] == [2048] * 7
    assert [deep.stage_chunk_elems(j) for j in (12, 13, 14, 15)] == [2048, 3072, 3072, 3072]   # 20, 18, 16, 14 bytes
    # an explicit size applies to every stage; a byte target scales all of them
    fixed = B.plan_for_workload(w, chunk_elems=2048)
    assert [fixed.stage_chunk_elems(j) for j in range(8)] == [2048] * 8 and fixed.n_chunks == 42272
    big = B.plan_for_workload(w, tuning=dict(chunk_bytes=96 * 1024))
    assert [big.stage_chunk_elems(j) for j in range(8)] == [4096] * 5 + [5120, 6144, 8192]
    assert plan.stage_chunk_elems(8) == -1 and plan.stage_n_chunks(-1) == -1


def test_minimal_ring_depth_is_paper_count(lib):
    """Stage j of a P-stage pipeline keeps P-j versions (T2 with one accumulation step)."""
    P = 5
    tau = [P - 1 - j for j in range(P)]
    plan, _ = _plan([[64]] * P, tau, R=B.FERRET_RING_DEPTH_MINIMAL)
    assert [plan.stage_ring_depth(j) for j in range(P)] == [P - j for j in range(P)]


def test_tuning_changes_slot_stride_only(lib):
    base, _ = _plan([[1000], [1000]], [1, 0], R=2)
    tuned, _ = _plan([[1000], [1000]], [1, 0], R=2, tuning=dict(slot_align_elems=1024, slot_skew_elems=32))
    assert base.stage_slot_stride(0) == 1024            # 1000 rounded up to the default 64
    assert tuned.stage_slot_stride(0) == 1024 + 32
    assert tuned.stage_numel(0) == base.stage_numel(0) == 1000
    assert tuned.flat_elems == base.flat_elems


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_benchmark_workload_plans(lib, idx):
    w = W.make_workload(idx)
    plan = B.plan_for_workload(w)
    assert plan.total_params == w.numel
    assert [plan.stage_params(j) for j in range(w.n_stages)] == w.stage_numel()
    # with every slot valid the step reads K'+1 versions per stage
    R = w.ring_depth
    plan.set_state([R - 1] * w.n_stages, [R] * w.n_stages)
    elt = 4 if w.precision == "f32" else 2
    want = 0
    for j, n in enumerate(w.stage_numel()):
        Kp = O.effective_iters(w.n_iters, w.staleness[j])
        assert plan.stage_effective_iters(j) == Kp
        per = elt * (Kp + 3) + (8 if w.precision == "bf16" else 0)
        want += per * n
    assert plan.step_bytes == want
    if idx == 4:
        assert want == 1_898_268_384            # the configuration the bandwidth target is quoted on


def test_read_slots_follow_segment_boundaries(lib):
    for tau in range(0, 9):
        for K in (-1, 0, 1, 2, 3, 4):
            for R in (tau + 1, tau + 3):
                plan, _ = _plan([[64]], [tau], K=K, R=R)
                for head in {0, R - 1, R // 2}:
                    plan.set_state([head], [R])
                    bounds = O.segment_boundaries(tau, K)      # [tau] when there is no iteration
                    want = [(head - (tau - s)) % R for s in bounds]
                    assert plan.stage_read_slots(0) == want
                    assert plan.stage_write_slot(0) == (head + 1) % R
                    # the slot written may coincide only with the oldest version of a full-depth window
                    if (head + 1) % R in want:
                        assert R == tau + 1 and want.index((head + 1) % R) == 0


def test_warmup_staleness_and_commit_rules(lib):
    plan, _ = _plan([[64]], [3], K=-1, R=4)
    heads, valid = plan.get_state()
    assert heads == [0] and valid == [0]
    assert plan.stage_write_slot(0) == 0
    # nothing pushed yet: a step is a state error, and so is a commit
    rc = lib.ferret_compensate_step(plan.handle, 16, 16, None, 0.5, 0.01, None, None, None, None)
    assert rc == B.FERRET_ESTATE and "no weight version" in B.last_error()
    rc = lib.ferret_push_version(plan.handle, 16, None, -1, None, None)
    assert rc == B.FERRET_ESTATE and "without a step" in B.last_error()
    for held in range(1, 6):
        plan.set_state([(held - 1) % 4], [min(held, 4)])
        assert plan.stage_effective_staleness(0) == min(3, held - 1)


def test_set_state_validation(lib):
    plan, _ = _plan([[64], [64]], [1, 0], R=2)
    with pytest.raises(B.FerretError) as e:
        plan.set_state([2, 0], [1, 1])
    assert e.value.status == B.FERRET_EINVAL
    with pytest.raises(B.FerretError):
        plan.set_state([0, 0], [3, 1])
    plan.set_state([1, 0], [2, 1])
    assert plan.get_state() == ([1, 0], [2, 1])


BAD_PLANS = [
    dict(tensors=[], n_stages=1, tau=[0]),
    dict(tensors=[(10, 0)], n_stages=0, tau=[]),
    dict(tensors=[(10, 0)], n_stages=B.FERRET_MAX_STAGES + 1, tau=[0] * (B.FERRET_MAX_STAGES + 1)),
    dict(tensors=[(0, 0)], n_stages=1, tau=[0]),
    dict(tensors=[(10, 1)], n_stages=2, tau=[0, 0]),                # stage 0 empty
    dict(tensors=[(10, 0), (10, 2)], n_stages=3, tau=[0, 0, 0]),    # stage 1 skipped
    dict(tensors=[(10, 1), (10, 0)], n_stages=2, tau=[0, 0]),       # decreasing
    dict(tensors=[(10, 0)], n_stages=2, tau=[0, 0]),                # last stage empty
    dict(tensors=[(10, 0)], n_stages=1, tau=[-1]),
    dict(tensors=[(10, 0)], n_stages=1, tau=[2], R=2),              # tau >= ring depth
    dict(tensors=[(10, 0)], n_stages=1, tau=[0], K=-2),
    dict(tensors=[(10, 0)], n_stages=1, tau=[0], R=-1),
    dict(tensors=[(10, 0)], n_stages=1, tau=[0], prec=7),
    dict(tensors=[(10, 0)], n_stages=1, tau=[0], chunk=1000),
    dict(tensors=[(10, 0)], n_stages=1, tau=[0], tuning=dict(slot_align_elems=100)),
    dict(tensors=[(10, 0)], n_stages=1, tau=[0], tuning=dict(slot_skew_elems=3)),
    dict(tensors=[(10, 0)], n_stages=1, tau=[0], tuning=dict(resident_cap=33)),
    dict(tensors=[(10, 0)], n_stages=1, tau=[0], tuning=dict(reserved=1)),
    dict(tensors=[(10, 0)], n_stages=1, tau=[0], tuning=dict(newest_from_master=1)),      # fp32 plan
    dict(tensors=[(10, 0)], n_stages=1, tau=[0], prec=1, tuning=dict(newest_from_master=2)),
]


@pytest.mark.parametrize("bad", BAD_PLANS)
def test_plan_rejects_bad_arguments(lib, bad):
    with pytest.raises(B.FerretError) as e:
        B.ferret_plan_buckets(bad["tensors"], bad["n_stages"], bad["tau"], bad.get("K", 1), bad.get("R", 1),
                              bad.get("prec", B.FERRET_F32), bad.get("chunk", 0), bad.get("tuning"))
    assert e.value.status == B.FERRET_EINVAL and e.value.message


def test_step_and_push_argument_errors(lib):
    plan, _ = _plan([[64]], [1], R=2)
    plan.set_state([0], [1])
    step = lib.ferret_compensate_step
    h = plan.handle
    assert step(None, 16, 16, None, 0.5, 0.01, None, None, None, None) == B.FERRET_EINVAL
    assert step(h, None, 16, None, 0.5, 0.01, None, None, None, None) == B.FERRET_EINVAL
    assert step(h, 16, None, None, 0.5, 0.01, None, None, None, None) == B.FERRET_EINVAL
    assert step(h, 24, 16, None, 0.5, 0.01, None, None, None, None) == B.FERRET_EINVAL     # misaligned ring
    assert "aligned" in B.last_error()
    assert step(h, 16, 16, 32, 0.5, 0.01, None, None, None, None) == B.FERRET_EINVAL       # master on fp32 plan
    assert step(h, 16, 16, None, 0.5, 0.01, 32, None, None, None) == B.FERRET_EINVAL       # norms without workspace
    push = lib.ferret_push_version
    assert push(None, 16, None, -1, 16, None) == B.FERRET_EINVAL
    assert push(h, 16, None, 5, 16, None) == B.FERRET_EINVAL
    assert push(h, None, None, -1, 16, None) == B.FERRET_EINVAL
    assert push(h, 16, None, -1, 8, None) == B.FERRET_EINVAL                               # misaligned src
    assert push(h, 16, 32, -1, 16, None) == B.FERRET_EINVAL                                # master on fp32 plan
    mixed, _ = _plan([[64]], [1], R=2, prec=B.FERRET_BF16_MASTER_F32)
    mixed.set_state([0], [1])
    assert step(mixed.handle, 16, 16, None, 0.5, 0.01, None, None, None, None) == B.FERRET_EINVAL
    assert "master" in B.last_error()
    assert lib.ferret_copy_bytes(16, 16, 8, None) == B.FERRET_EINVAL
    assert lib.ferret_copy_bytes(16, 16, 0, None) == B.FERRET_OK


def test_tuning_validation(lib):
    def bad(**tuning):
        with pytest.raises(B.FerretError) as e:
            _plan([[4096]], [1], R=2, prec=tuning.pop("prec", B.FERRET_F32), chunk=tuning.pop("chunk", 0), tuning=tuning)
        assert e.value.status == B.FERRET_EINVAL
        return e.value.message
    assert "resident_cap" in bad(resident_cap=1)              # one workgroup cannot hold more than 64 of 160 KiB
    assert "resident_cap" in bad(resident_cap=33)
    assert "cache_policy" in bad(cache_policy=3)
    assert "xcd_group" in bad(xcd_group=-1) and "xcd_group" in bad(xcd_group=5000)
    assert "chunk_bytes" in bad(chunk_bytes=-1)
    assert "not both" in bad(chunk_bytes=4096, chunk=1024)
    assert "persistent" in bad(newest_from_master=1, blocks_per_cu=2, prec=B.FERRET_BF16_MASTER_F32)
    assert "reserved" in bad(reserved=1)
    with pytest.raises(ValueError):
        _plan([[4096]], [1], R=2, tuning=dict(no_such_field=1))
    for ok in (dict(resident_cap=2), dict(resident_cap=-1), dict(cache_policy=1), dict(cache_policy=2),
               dict(chunk_bytes=1), dict(chunk_bytes=1 << 30), dict(xcd_group=1), dict(xcd_group=16)):
        plan, _ = _plan([[4096]], [1], R=2, tuning=ok)
        assert plan.n_chunks >= 1 and plan.stage_chunk_elems(0) % 1024 == 0


def test_noalloc_step_rejects_plans_beyond_its_scratch(lib):
    """The entry point that allocates nothing holds partial sums for a fixed number of chunks; a plan with more
    is refused before any device call (so this runs without a GPU), with the same argument checks otherwise."""
    fn = lib.ferret_compensate_step_noalloc
    n = (B.FERRET_NOALLOC_MAX_CHUNKS + 1) * 1024
    plan, _ = _plan([[n]], [0], R=1, chunk=1024)
    plan.set_state([0], [1])
    assert plan.n_chunks == B.FERRET_NOALLOC_MAX_CHUNKS + 1
    assert fn(plan.handle, 16, 16, None, 0.5, 0.01, None, None, None) == B.FERRET_EINVAL
    assert "chunks" in B.last_error() and str(B.FERRET_NOALLOC_MAX_CHUNKS) in B.last_error()
    header = open(os.path.join(ROOT, "include", "ferret.h")).read()
    assert re.search(r"#define\s+FERRET_NOALLOC_MAX_CHUNKS\s+%d\b" % B.FERRET_NOALLOC_MAX_CHUNKS, header)
    small, _ = _plan([[64]], [1], R=2)
    small.set_state([0], [1])
    assert fn(None, 16, 16, None, 0.5, 0.01, None, None, None) == B.FERRET_EINVAL
    assert fn(small.handle, 24, 16, None, 0.5, 0.01, None, None, None) == B.FERRET_EINVAL       # misaligned ring
    assert fn(small.handle, 16, 16, 32, 0.5, 0.01, None, None, None) == B.FERRET_EINVAL         # master on fp32 plan


def test_queries_on_null_or_out_of_range(lib):
    assert lib.ferret_plan_n_stages(None) == -1
    assert lib.ferret_plan_ring_bytes(None) == 0
    plan, _ = _plan([[64]], [0], R=1)
    assert plan.stage_numel(3) == -1 and plan.tensor_offset(-1) == -1
    lib.ferret_plan_destroy(None)


def test_adaptive_step_argument_errors(lib):
    plan, _ = _plan([[64]], [1], R=2)
    plan.set_state([0], [1])
    fn = lib.ferret_compensate_step_adaptive
    ad = B.ferret_adaptive(16, 16, 16, 0.9, 1e-3)
    import ctypes
    assert fn(plan.handle, 16, 16, None, None, 0.01, None, None, 16, None) == B.FERRET_EINVAL      # no state
    assert fn(plan.handle, 16, 16, None, ctypes.byref(ad), 0.01, None, None, None, None) == B.FERRET_EINVAL  # no workspace
    bad = B.ferret_adaptive(16, 16, 16, 1.0, 1e-3)
    assert fn(plan.handle, 16, 16, None, ctypes.byref(bad), 0.01, None, None, 16, None) == B.FERRET_EINVAL
    assert "alpha" in B.last_error()
    bad = B.ferret_adaptive(16, 24, 16, 0.9, 1e-3)
    assert fn(plan.handle, 16, 16, None, ctypes.byref(bad), 0.01, None, None, 16, None) == B.FERRET_EINVAL
    bad = B.ferret_adaptive(16, 16, 16, 0.9, -1.0)
    assert fn(plan.handle, 16, 16, None, ctypes.byref(bad), 0.01, None, None, 16, None) == B.FERRET_EINVAL
    zero, _ = _plan([[64]], [1], K=0, R=2)
    zero.set_state([0], [1])
    assert fn(zero.handle, 16, 16, None, ctypes.byref(ad), 0.01, None, None, 16, None) == B.FERRET_EINVAL
    assert "n_iters" in B.last_error()


def test_accumulate_step_argument_errors(lib):
    import ctypes
    plan, _ = _plan([[64], [64]], [2, 0], R=3)
    plan.set_state([0, 0], [1, 1])
    fn = lib.ferret_accumulate_step
    mode = (ctypes.c_int32 * 2)(2, 1)
    ok = B.ferret_accumulate(16, 1.0, mode, None)
    assert fn(plan.handle, 16, 16, None, None, 0.5, 0.01, None, None, None, None) == B.FERRET_EINVAL
    bad = B.ferret_accumulate(None, 1.0, mode, None)
    assert fn(plan.handle, 16, 16, None, ctypes.byref(bad), 0.5, 0.01, None, None, None, None) == B.FERRET_EINVAL
    bad = B.ferret_accumulate(16, 1.0, (ctypes.c_int32 * 2)(3, 0), None)
    assert fn(plan.handle, 16, 16, None, ctypes.byref(bad), 0.5, 0.01, None, None, None, None) == B.FERRET_EINVAL
    assert "mode" in B.last_error()
    bad = B.ferret_accumulate(16, 1.0, mode, (ctypes.c_int32 * 2)(3, 0))
    assert fn(plan.handle, 16, 16, None, ctypes.byref(bad), 0.5, 0.01, None, None, None, None) == B.FERRET_EINVAL
    assert "staleness" in B.last_error()
    assert ok.scale == 1.0


def test_oracle_and_product_do_not_reach_into_each_other():
    """The oracle is test infrastructure: nothing in the package (sources included) names it, and nothing under
    oracle/ names the package or its C sources."""
    pkg = os.path.join(ROOT, "paper_2503_12053_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
                assert "ferret_oracle" not in text and "oracle/" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2503_12053_amd" not in text and "ferret_internal" not in text and "include/ferret" not in text, f
