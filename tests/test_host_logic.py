"""Host logic of libms (no GPU): symbols, op descriptors, space, sampler, mutation, text form,
validator, interpreter coverage."""
import ctypes as C
import collections
import math
import os
import re

import numpy as np
import pytest

from oracle import oracle as O
from paper_2205_13603_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "ms.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ms_[a-z0-9_]+)\s*\(", hdr))
    declared -= {n for n in declared if re.search(r"typedef[^;]*\(\s*\*\s*%s\s*\)" % n, hdr)}
    assert declared, "no declarations found"
    L = B.lib()
    for name in sorted(declared):
        assert hasattr(L, name), "libms.so does not export %s" % name
    assert declared == set(B.SYMBOLS), (declared ^ set(B.SYMBOLS))
    assert L.ms_version() == 3


def test_struct_sizes_match_header():
    # computed from the header's field lists (natural alignment)
    assert C.sizeof(B.ms_decision) == 16 + 8 * B.MAX_FACTORS
    assert C.sizeof(B.ms_trace) == 8 + B.MAX_SLOTS * C.sizeof(B.ms_decision)
    assert C.sizeof(B.ms_op_desc) == 8 * 4 + 8 * 8 + 3 * 8 + 3 * 8
    assert C.sizeof(B.ms_slot) == 8 + 16 + 8 + 8 + 8 * B.MAX_CANDS + 4 * B.MAX_CANDS + 8 + 8 * B.MAX_CANDS


def test_op_loops_and_work():
    op = B.gemm_op(128, 128, 128, "f32")
    assert op.loops() == [("i", 128, False), ("j", 128, False), ("k", 128, True)]
    assert op.work() == (4194304.0, 196608.0)
    op = B.gemm_op(1024, 1024, 1024, "f16")
    assert op.work() == (2147483648.0, 6291456.0)
    op = B.conv2d_op(1, 56, 56, 64, 64, 3, 3, stride=1, pad=1)
    assert op.loops() == [("i", 3136, False), ("j", 64, False), ("k", 576, True)]
    f, b = op.work()
    assert f == 231211008.0 and b == 401408 + 73728 + 256 + 401408
    op = B.bmm_op(12, 128, 128, 64, True, "f16")
    assert op.work() == (25165824.0, 786432.0)
    d = op.desc()
    assert list(d.a_strides) == [128 * 64, 64, 1] and list(d.b_strides) == [128 * 64, 1, 64]
    op = B.bmm_op(12, 128, 64, 128, False, "f16")
    assert op.work() == (25165824.0, 786432.0)
    op = B.gemm_op(512, 512, 512, "i8")
    assert op.work() == (268435456.0, 1572864.0)
    op = B.dwconv2d_op(1, 112, 112, 32)
    assert op.work() == (7225344.0, 3212416.0)
    assert [l[0] for l in op.loops()] == ["n", "i", "j", "c", "kh", "kw"]
    op = B.dwconv2d_op(1, 56, 56, 144, stride=2)
    assert op.work() == (2032128.0, 2263104.0)
    assert op.tensor_bytes(-1) == 28 * 28 * 144 * 4


def test_op_errors_do_not_abort():
    with pytest.raises(B.MsError) as e:
        B.gemm_op(0, 4, 4)
    assert e.value.code == B.MS_ERR_BAD_ARG
    with pytest.raises(B.MsError) as e:
        B.gemm_op(4, 4, 4, "i8", "f16")
    assert e.value.code == B.MS_ERR_UNSUPPORTED
    with pytest.raises(B.MsError) as e:
        B.Op(17, "f32", "f32", [1, 1, 1])
    assert e.value.code == B.MS_ERR_BAD_ARG
    assert B.lib().ms_op_create(None, None) == B.MS_ERR_BAD_ARG
    B.lib().ms_op_destroy(None)
    B.lib().ms_variant_destroy(None)
    with pytest.raises(B.MsError) as e:
        B.conv2d_op(1, 8, 8, 4, 4, 3, 3, in_dtype="f32", out_dtype="f32").space()
    assert e.value.code == B.MS_ERR_UNSUPPORTED


def slot_names(sp):
    return [sp.slots[i].name.decode() for i in range(sp.n_slots)]


def test_space_composition_by_flags():
    op = B.gemm_op(128, 128, 128, "f32")
    assert slot_names(op.space(B.SPACE_UNROLL)) == ["i", "j", "k", "unroll"]
    assert op.space(B.SPACE_UNROLL).family == B.FAM_GEMM_ALU
    assert slot_names(op.space(0)) == ["i", "j", "k"]
    sp = op.space()
    assert slot_names(sp) == ["i", "j", "k", "unroll", "cache_read", "vectorize", "vectorize_b", "storage_align", "reorder"]
    un = sp.slots[3]
    assert [un.candidates[i] for i in range(un.n_candidates)] == [0, 16, 64]
    op = B.gemm_op(1024, 1024, 1024, "f16")
    sp = op.space()
    assert sp.family == B.FAM_GEMM_MFMA and slot_names(sp)[0] == "tensorize"
    t = sp.slots[0]
    assert [t.candidates[i] for i in range(t.n_candidates)] == [161616, 323208, 161632, 323216]
    assert sp.slots[1].depends_on == 0 and [sp.slots[1].extent_by_choice[c] for c in range(4)] == [64, 32, 64, 32]
    assert [sp.slots[3].extent_by_choice[c] for c in range(4)] == [64, 128, 32, 64]
    assert op.space(B.SPACE_DEFAULT & ~B.SPACE_TENSORIZE).family == B.FAM_GEMM_ALU
    op = B.dwconv2d_op(1, 112, 112, 32)
    assert slot_names(op.space()) == ["i", "j", "c", "unroll", "cache_read", "reorder"]
    # fp32 on the matrix cores is opt-in; all-ones masks (earlier tuning records) mean the default set
    op = B.gemm_op(128, 128, 128, "f32")
    assert op.space().family == B.FAM_GEMM_ALU and op.space(0xFFFFFFFF).family == B.FAM_GEMM_ALU
    sp = op.space(B.SPACE_DEFAULT | B.SPACE_TENSORIZE_F32)
    assert sp.family == B.FAM_GEMM_MFMA
    assert [sp.slots[0].candidates[i] for i in range(sp.slots[0].n_candidates)] == [161604, 323202]
    assert [sp.slots[1].extent_by_choice[c] for c in range(2)] == [8, 4] and [sp.slots[3].extent_by_choice[c] for c in range(2)] == [32, 64]
    assert B.dwconv2d_op(1, 8, 8, 4).space(B.SPACE_DEFAULT | B.SPACE_TENSORIZE_F32).family == B.FAM_DWCONV
    assert B.gemm_op(64, 64, 64, "f16").space(B.SPACE_DEFAULT | B.SPACE_TENSORIZE_F32).flags == B.SPACE_DEFAULT & ~B.SPACE_COMPUTE_AT


def test_space_size_matches_closed_form():
    op = B.gemm_op(128, 128, 128, "f32")
    assert abs(B.space_log10_size(op.space(B.SPACE_UNROLL)) - math.log10(120 ** 3 * 3)) < 1e-9


@pytest.mark.parametrize("extent", [128, 56, 144, 3136, 12])
def test_sampler_support_and_uniformity(extent):
    """sample-perfect-tile: only members of the brute-force support, all of them reached, uniform."""
    op = B.gemm_op(extent, 4, 4, "f32")
    sp = op.space(0)
    support = {tuple(t) for t in O.perfect_tiles(extent, 4).tolist()}
    n = len(support)
    draws = 60 * n
    cnt = collections.Counter()
    for idx in range(draws):
        t = B.trace_sample(sp, 11, idx)
        f = tuple(t.d[0].v[k] for k in range(4))
        assert f in support
        cnt[f] += 1
    assert set(cnt) == support
    exp = draws / n
    chi2 = sum((c - exp) ** 2 / exp for c in cnt.values())
    # chi-square with n-1 dof: mean n-1, sd sqrt(2(n-1)); 6 sigma
    assert chi2 < (n - 1) + 6 * math.sqrt(2 * (n - 1)), (chi2, n)


def test_sampler_is_deterministic_and_seed_dependent():
    op = B.gemm_op(1024, 1024, 1024, "f16")
    sp = op.space()
    a = [B.trace_sample(sp, 5, i).decisions() for i in range(20)]
    b = [B.trace_sample(sp, 5, i).decisions() for i in range(20)]
    c = [B.trace_sample(sp, 6, i).decisions() for i in range(20)]
    assert a == b and a != c and len({str(x) for x in a}) > 15


def test_categorical_frequencies():
    op = B.gemm_op(128, 128, 128, "f32")
    sp = op.space(B.SPACE_UNROLL)
    cnt = collections.Counter(B.trace_sample(sp, 3, i).d[3].v[0] for i in range(3000))
    assert set(cnt) == {0, 1, 2} and all(abs(c - 1000) < 150 for c in cnt.values())


def test_dependent_tile_extents_follow_the_tensorize_decision():
    op = B.gemm_op(1024, 1024, 1024, "f16")
    sp = op.space()
    seen = set()
    for i in range(200):
        t = B.trace_sample(sp, 9, i)
        code = sp.slots[0].candidates[t.d[0].v[0]]
        m, n, k = code // 10000, code // 100 % 100, code % 100
        seen.add(code)
        assert math.prod(t.d[1].v[q] for q in range(4)) == 1024 // m
        assert math.prod(t.d[2].v[q] for q in range(4)) == 1024 // n
        assert math.prod(t.d[3].v[q] for q in range(4)) == 1024 // k
    assert len(seen) == 4


def test_mutation_changes_one_decision_and_keeps_products():
    op = B.gemm_op(1024, 1024, 1024, "f16")
    sp = op.space()
    t = B.trace_sample(sp, 1, 0)
    changed_slots = collections.Counter()
    for s in range(400):
        m = B.trace_mutate(sp, t, s)
        a, b = t.decisions(), m.decisions()
        diff = [i for i in range(len(a)) if a[i] != b[i]]
        assert diff, "mutation returned the same trace"
        if diff[0] == 0:  # tensorize changed: dependent tiles are redrawn for the new unit
            assert set(diff) <= {0, 1, 2, 3}
        else:
            assert len(diff) == 1
            i = diff[0]
            if sp.slots[i].kind == B.SLOT_PERFECT_TILE:
                assert math.prod(a[i][1]) == math.prod(b[i][1])
                assert sum(1 for x, y in zip(a[i][1], b[i][1]) if x != y) == 2
        changed_slots[diff[0]] += 1
        code = sp.slots[0].candidates[m.d[0].v[0]]
        for l, u in zip((1, 2, 3), (code // 10000, code // 100 % 100, code % 100)):
            assert math.prod(m.d[l].v[q] for q in range(4)) * u == 1024
    assert len(changed_slots) == sp.n_slots


def test_text_round_trip():
    for op in [B.gemm_op(128, 128, 128, "f32"), B.gemm_op(1024, 1024, 1024, "f16"), B.dwconv2d_op(1, 112, 112, 32)]:
        sp = op.space()
        for i in range(10):
            t = B.trace_sample(sp, 2, i)
            text = B.trace_to_text(op, sp, t)
            assert text.count("sample-") == sp.n_slots
            back = B.trace_from_text(sp, text)
            assert back.decisions() == t.decisions()
            assert bytes(back) == bytes(t)


def test_text_worked_example_split():
    """The split of Section 3.1's figure: loop of 1024 into extents 32, 8, 4 (here with a leading 1)."""
    op = B.gemm_op(1024, 4, 4, "f32")
    sp = op.space(0)
    t = B.make_trace(sp, [[1, 32, 8, 4], [1, 1, 4, 1], [1, 1, 4, 1]])
    p = B.trace_validate(op, sp, t)
    assert list(p.ti) == [1, 32, 8, 4] and p.block_m == 1024 and p.threads == 8 * 4
    text = B.trace_to_text(op, sp, t)
    assert "split(loop=i, factors=[1, 32, 8, 4])" in text
    cov = B.variant_coverage(op, p, 1024 * 4)
    assert np.all(cov == 1)


def test_text_errors():
    op = B.gemm_op(128, 128, 128, "f32")
    sp = op.space(B.SPACE_UNROLL)
    t = B.trace_sample(sp, 0, 0)
    text = B.trace_to_text(op, sp, t)
    lines = text.splitlines()
    trunc = "\n".join(l for l in lines if "slot=unroll" not in l)
    with pytest.raises(B.MsError) as e:
        B.trace_from_text(sp, trunc)
    assert e.value.code == B.MS_ERR_INVALID_TRACE and "truncated" in str(e.value)
    swapped = text.replace("slot=i,", "slot=q,")
    with pytest.raises(B.MsError):
        B.trace_from_text(sp, swapped)


def test_validator_rejections():
    op = B.gemm_op(128, 128, 128, "f32")
    sp = op.space()

    def mk(i, j, k, unroll=0, cache=1, vec=1, vec_b=1, pad=0, reorder=0):
        return B.make_trace(sp, [i, j, k, [unroll], [cache], [vec], [vec_b], [pad], [reorder]])

    ok = mk([4, 2, 8, 2], [4, 2, 16, 1], [4, 4, 4, 2])
    p = B.trace_validate(op, sp, ok)
    assert p.threads == 128 and p.block_m == 32 and p.block_n == 32 and p.block_k == 32 and p.grid[0] == 16
    assert p.lds_bytes == 4 * (32 * 32 + 32 * 32) and p.acc_per_thread == 8

    def rejected(t, word):
        with pytest.raises(B.MsError) as e:
            B.trace_validate(op, sp, t)
        assert e.value.code == B.MS_ERR_INVALID_TRACE and word in str(e.value), str(e.value)

    rejected(mk([4, 2, 8, 4], [4, 2, 16, 1], [4, 4, 4, 2]), "multiply to")          # product != extent
    rejected(mk([1, 1, 128, 1], [1, 1, 128, 1], [4, 4, 4, 2]), "threads per workgroup")  # 16384 threads
    rejected(mk([1, 16, 1, 8], [1, 16, 1, 8], [128, 1, 1, 1]), "accumulators per lane")
    rejected(mk([1, 2, 32, 2], [1, 2, 32, 2], [1, 1, 128, 1], cache=2), "LDS tile needs")  # 2*(128*128*2)*4 = 256 KiB
    rejected(mk([4, 2, 8, 2], [4, 2, 16, 1], [4, 4, 4, 2], cache=0, pad=1), "nothing to pad")
    bad = ok.copy()
    bad.d[0].v[0] = 0
    rejected(bad, "factor 0 is 0")
    bad = ok.copy()
    bad.d[3].v[0] = 7
    rejected(bad, "outside")
    bad = ok.copy()
    bad.n = 5
    rejected(bad, "truncated")
    bad = ok.copy()
    bad.d[1].slot_id = 99
    rejected(bad, "slot id")
    # vector width must divide the contiguous tile extent: BK = 2 with 4-wide loads of A; BN = 2 for B
    rejected(mk([4, 2, 8, 2], [4, 2, 16, 1], [64, 1, 1, 2], vec=4), "vector width")
    rejected(mk([4, 2, 8, 2], [64, 1, 2, 1], [4, 4, 4, 2], vec_b=4), "vector width")
    # forced smaller hardware limits reject what passed before, and are restorable
    lim = B.get_limits()
    small = B.ms_limits(64, 4096, 16, 64, 2)
    B.set_limits(small)
    try:
        rejected(ok, "threads per workgroup")
    finally:
        B.set_limits(lim)
    B.trace_validate(op, sp, ok)


def test_validator_mfma_rules():
    op = B.gemm_op(1024, 1024, 1024, "f16")
    sp = op.space()

    def mk(mfma, i, j, k, unroll=0, cache=2, vec=8, vec_b=8, pad=0, reorder=0, cw=0):
        return B.make_trace(sp, [[mfma], i, j, k, [unroll], [cache], [vec], [vec_b], [pad], [reorder], [cw]])

    p = B.trace_validate(op, sp, mk(323216, [4, 2, 2, 2], [4, 2, 2, 2], [16, 1, 2, 2]))
    assert (p.block_m, p.block_n, p.block_k) == (256, 256, 64) and p.waves == 4 and p.threads == 256
    assert p.acc_per_thread == 256 and p.lds_bytes == 2 * (64 // 8) * (256 * 16 + 256 * 16)
    with pytest.raises(B.MsError) as e:
        B.trace_validate(op, sp, mk(323216, [1, 1, 32, 1], [32, 1, 1, 1], [16, 1, 2, 2]))
    assert "wavefronts" in str(e.value)
    with pytest.raises(B.MsError) as e:
        B.trace_validate(op, sp, mk(323216, [2, 4, 1, 4], [2, 4, 1, 4], [16, 1, 2, 2]))
    assert "accumulators" in str(e.value)
    with pytest.raises(B.MsError) as e:  # i tile counted for 16-wide intrinsic but 32-wide chosen
        B.trace_validate(op, sp, mk(323216, [4, 2, 2, 4], [4, 2, 2, 2], [16, 1, 2, 2]))
    assert "multiply to" in str(e.value)


def test_validator_conv_compute_location_rules():
    """sample-compute-location for conv2d: LDS footprints of the resident patch / weights and the constraints
    each location puts on the other decisions (all checked on the host)."""
    op = B.conv2d_op(1, 56, 56, 64, 64, 3, 3, stride=1, pad=1)
    sp = op.space()
    assert slot_names(sp)[-1] == "compute_at"

    def mk(ca, mfma=161632, i=(14, 7, 2, 1), j=(1, 2, 2, 1), k=(9, 1, 2, 1), unroll=64, cache=2, vec=8, vec_b=8, pad=1, reorder=0, cw=1):
        return B.make_trace(sp, [[mfma], list(i), list(j), list(k), [unroll], [cache], [vec], [vec_b], [pad], [reorder], [cw], [ca]])

    planes_b = (64 // 8) * (64 * 16 + 16)             # one k step of the weights: 8 k-group planes of 64 fragments + pad
    patch = 6 * 58 * (64 * 2 + 16)                    # 4 output rows -> 6 input rows x (56 + 2) columns x padded pixel
    ctile = 224 * (64 * 2 + 16)
    p0 = B.trace_validate(op, sp, mk(0))
    assert p0.compute_at == 0 and p0.threads == 256
    p1 = B.trace_validate(op, sp, mk(1))
    assert p1.lds_bytes == 2 * planes_b + patch and p1.grid[0] == 14
    p2 = B.trace_validate(op, sp, mk(2))
    assert p2.lds_bytes == 9 * planes_b + patch + ctile and p2.threads == 256
    p3 = B.trace_validate(op, sp, mk(3))
    assert p3.waves == 8 and p3.threads == 512 and p3.lds_bytes == p2.lds_bytes  # four helper wavefronts
    p4 = B.trace_validate(op, sp, mk(4))
    assert p4.lds_bytes == planes_b + patch + ctile
    assert len({p.key for p in (p0, p1, p2, p3, p4)}) == 5
    for ca, kw, needle in [(1, dict(cache=4), "cache_read"), (2, dict(cache=3), "cache_read"), (2, dict(reorder=2), "reorder"),
                           (3, dict(cw=0), "cache_write"), (3, dict(cache=1), "cache_read"),
                           (4, dict(i=(7, 14, 2, 1), j=(1, 4, 1, 1)), "weights in registers"),
                           (2, dict(i=(7, 14, 2, 1), k=(1, 9, 2, 1)), "LDS")]:
        with pytest.raises(B.MsError) as e:
            B.trace_validate(op, sp, mk(ca, **kw))
        assert needle in str(e.value), (ca, kw, str(e.value))
    # a 16-pixel tile of a 12-wide image starts in the middle of a row: 3 output rows, 5 patch rows; Cin = 24 is not
    # a multiple of the 32-deep intrinsic
    op2 = B.conv2d_op(1, 12, 12, 32, 32, 3, 3, stride=1, pad=1)
    sp2 = op2.space()
    t = B.make_trace(sp2, [[161632], [9, 1, 1, 1], [1, 2, 1, 1], [9, 1, 1, 1], [0], [1], [8], [8], [0], [0], [0], [1]])
    assert B.trace_validate(op2, sp2, t).lds_bytes == 1 * (32 // 8) * (32 * 16) + 5 * 14 * 64
    op3 = B.conv2d_op(1, 12, 12, 16, 32, 3, 3, stride=1, pad=1)
    sp3 = op3.space()
    cands = [sp3.slots[0].candidates[i] for i in range(sp3.slots[0].n_candidates)]
    assert 161616 in cands
    t = B.make_trace(sp3, [[161616], [9, 1, 1, 1], [1, 2, 1, 1], [9, 1, 1, 1], [0], [1], [8], [8], [0], [0], [0], [1]])
    assert B.trace_validate(op3, sp3, t).compute_at == 1
    assert 161632 in cands
    if True:
        # K = 144 is rounded up to 160 for the 32-deep intrinsic (5 k steps, zero padded by the im2col loader only)
        t = B.make_trace(sp3, [[161632], [9, 1, 1, 1], [1, 2, 1, 1], [5, 1, 1, 1], [0], [1], [8], [8], [0], [0], [0], [1]])
        with pytest.raises(B.MsError) as e:
            B.trace_validate(op3, sp3, t)
        assert "Cin" in str(e.value) and "compute_at must be 0" in str(e.value)
        t = B.make_trace(sp3, [[161632], [9, 1, 1, 1], [1, 2, 1, 1], [5, 1, 1, 1], [0], [1], [8], [8], [0], [0], [0], [0]])
        assert B.trace_validate(op3, sp3, t).block_k == 32


CONFIG_OPS = [
    lambda: B.gemm_op(128, 128, 128, "f32"),
    lambda: B.gemm_op(256, 128, 64, "f16"),
    lambda: B.bmm_op(3, 128, 128, 64, True, "f16"),
    lambda: B.gemm_op(128, 64, 128, "i8"),
    lambda: B.conv2d_op(1, 28, 28, 16, 32, 3, 3, stride=1, pad=1),
    lambda: B.dwconv2d_op(1, 28, 28, 12),
    lambda: B.dwconv2d_op(2, 14, 14, 18, stride=2),
]


@pytest.mark.parametrize("mk", CONFIG_OPS)
def test_interpreter_covers_every_output_once(mk):
    """The split/bind structure derived from any valid trace tiles the output exactly once."""
    op = mk()
    sp = op.space()
    elems = op.tensor_bytes(-1) // {B.F32: 4, B.F16: 2, B.BF16: 2, B.I32: 4}[op.desc().out_dtype]
    for idx in range(25):
        t = B.trace_sample_valid(op, sp, 21, idx)
        p = B.trace_validate(op, sp, t)
        cov = B.variant_coverage(op, p, elems)
        assert cov.min() == 1 and cov.max() == 1, t.decisions()


# ---------------------------------------------------------------- softmax / norm (row reductions)

def test_reduce_ops_descriptor_loops_and_work():
    op = B.softmax_op(2, 48, 96, "f16")
    assert op.loops() == [("i", 96, False), ("k", 96, True)]
    assert op.tensor_bytes(0) == 2 * 48 * 96 * 2 and op.tensor_bytes(-1) == 2 * 48 * 96 * 2
    assert op.work()[1] == 2 * 48 * 96 * 4
    op = B.norm_op(3, 16, 20, "bf16")
    assert op.loops() == [("i", 3, False), ("k", 320, True)]
    assert op.tensor_bytes(0) == 3 * 320 * 2 and op.tensor_bytes(-1) == 3 * 4
    assert op.work() == (2.0 * 3 * 320, 3 * 320 * 2 + 12.0)
    with pytest.raises(B.MsError):
        B.Op(B.OP_NORM, "f32", "f16", [1, 4, 4])       # the norm is written in fp32
    with pytest.raises(B.MsError):
        B.Op(B.OP_SOFTMAX, "i8", "i32", [1, 4, 4])
    with pytest.raises(B.MsError):
        B.Op(B.OP_SOFTMAX, "f32", "f32", [1, 4, 4], stride=1)


def test_reduce_space_coverage_and_text_round_trip():
    for op, elems in ((B.softmax_op(1, 256, 256), 65536), (B.softmax_op(3, 20, 96, "f16"), 5760), (B.norm_op(6, 32, 24), 6)):
        sp = op.space()
        assert sp.family == B.FAM_REDUCE
        names = [sp.slots[i].name.decode() for i in range(sp.n_slots)]
        assert names[:2] == ["i", "k"] and (names[2:] == ["cache_read"]) == (elems != 6)
        for idx in range(20):
            t = B.trace_sample_valid(op, sp, 33, idx)
            p = B.trace_validate(op, sp, t)
            assert p.threads == p.ti[2] * p.tk[2] and p.threads % 64 == 0 and p.grid[0] == p.ti[0]
            cov = B.variant_coverage(op, p, elems)
            assert cov.min() == 1 and cov.max() == 1, t.decisions()
            text = B.trace_to_text(op, sp, t)
            assert "cross-thread reduction over %d lanes" % p.tk[2] in text
            assert B.trace_from_text(sp, text).decisions() == t.decisions()
    # without the cache-read module the softmax space has only the two tile slots
    assert B.softmax_op(1, 8, 64).space(0).n_slots == 2


def test_reduce_validator_rejections():
    op = B.softmax_op(1, 64, 256)
    sp = op.space()

    def why(vals):
        with pytest.raises(B.MsError) as e:
            B.trace_validate(op, sp, B.make_trace(sp, vals))
        assert e.value.code == B.MS_ERR_INVALID_TRACE
        return str(e.value)

    assert "at most 16 bytes" in why([[1, 1, 64, 1], [1, 1, 32, 8], [0]])
    assert "power of two" not in why([[1, 1, 64, 1], [1, 1, 32, 8], [0]])
    assert "whole number of wavefronts" in why([[32, 1, 2, 1], [4, 4, 16, 1], [0]])
    assert "threads per workgroup" in why([[1, 1, 64, 1], [2, 1, 32, 4], [0]])
    assert "register budget" in why([[1, 1, 8, 8], [8, 4, 8, 1], [1]])
    op3 = B.softmax_op(1, 64, 96)
    sp3 = op3.space()
    with pytest.raises(B.MsError) as e:
        B.trace_validate(op3, sp3, B.make_trace(sp3, [[1, 1, 64, 1], [1, 8, 12, 1], [0]]))
    assert "power of two" in str(e.value)
    opn = B.norm_op(1, 256, 256)
    spn = opn.space()
    with pytest.raises(B.MsError) as e:
        B.trace_validate(opn, spn, B.make_trace(spn, [[1, 1, 1, 1], [512, 2, 16, 4]]))
    assert "one wavefront per row" in str(e.value)


def test_transposed_conv_descriptor_and_space():
    op = B.conv2d_transposed_op(1, 4, 4, 512, 256, 4, 4, stride=2, pad=1)
    assert op.loops() == [("i", 64, False), ("j", 256, False), ("k", 8192, True)]      # 8 x 8 output pixels
    assert op.tensor_bytes(-1) == 64 * 256 * 2 and op.tensor_bytes(0) == 16 * 512 * 2 and op.tensor_bytes(1) == 8192 * 256 * 2
    assert op.work()[0] == 2.0 * 16 * 8192 * 256
    sp = op.space()
    assert sp.family == B.FAM_GEMM_MFMA
    assert "compute_at" not in [sp.slots[i].name.decode() for i in range(sp.n_slots)]
    t = B.trace_sample_valid(op, sp, 2, 0)
    p = B.trace_validate(op, sp, t)
    assert p.compute_at == 0
    cov = B.variant_coverage(op, p, 64 * 256)
    assert cov.min() == 1 and cov.max() == 1
    assert "op=conv2d_transposed_nhwc" in B.trace_to_text(op, sp, t)
    with pytest.raises(B.MsError):
        B.Op(B.OP_CONV2D_TRANSPOSED_NHWC, "f16", "f16", [1, 4, 4, 8, 8, 3, 3], stride=1, pad=0, dilation=2)
    with pytest.raises(B.MsError):
        B.conv2d_transposed_op(1, 1, 1, 8, 8, 2, 2, stride=1, pad=1)   # empty output


def test_grouped_conv_descriptor_space_and_coverage():
    op = B.conv2d_op(1, 56, 56, 64, 128, 3, 3, stride=2, pad=1, groups=4)
    assert op.loops() == [("g", 4, False), ("i", 784, False), ("j", 32, False), ("k", 144, True)]
    assert op.tensor_bytes(1) == 3 * 3 * 16 * 128 * 2 and op.tensor_bytes(-1) == 784 * 128 * 2 and op.tensor_bytes(2) == 128 * 4
    assert op.work()[0] == 2.0 * 784 * 128 * 144
    sp = op.space()
    ca = [sp.slots[i] for i in range(sp.n_slots) if sp.slots[i].name == b"compute_at"][0]
    assert list(ca.weight)[:5] == [1, 1, 1, 1, 1]      # 16 channels per group: every compute location
    seen = set()
    for idx in range(10):
        t = B.trace_sample_valid(op, sp, 7, idx)
        p = B.trace_validate(op, sp, t)
        assert p.grid[2] == 4
        seen.add(p.compute_at)
        cov = B.variant_coverage(op, p, 784 * 128)
        assert cov.min() == 1 and cov.max() == 1
    with pytest.raises(B.MsError):
        B.conv2d_op(1, 8, 8, 30, 64, 3, 3, groups=4)          # 4 does not divide 30
    with pytest.raises(B.MsError):
        B.Op(B.OP_CONV2D_TRANSPOSED_NHWC, "f16", "f16", [1, 4, 4, 16, 16, 2, 2, 2], stride=1, pad=0)
    # a dense convolution is unchanged by the new field: same kernel key with groups 0 and 1
    d0, d1 = B.conv2d_op(1, 8, 8, 16, 32, 3, 3, pad=1), B.conv2d_op(1, 8, 8, 16, 32, 3, 3, pad=1, groups=1)
    s0 = d0.space()
    t = B.trace_sample_valid(d0, s0, 1, 0)
    assert B.trace_validate(d0, s0, t).key == B.trace_validate(d1, d1.space(), t).key


def test_conv1d_descriptor_runs_on_the_conv2d_space():
    op = B.conv1d_op(1, 256, 64, 128, 3, stride=2, pad=1)
    assert op.loops() == [("i", 128, False), ("j", 128, False), ("k", 192, True)]        # OL = 128
    d = op.desc()
    assert d.kind == B.OP_CONV1D_NWC and list(d.dims)[:5] == [1, 256, 64, 128, 3]        # the descriptor as given
    assert op.tensor_bytes(0) == 256 * 64 * 2 and op.tensor_bytes(1) == 3 * 64 * 128 * 2 and op.tensor_bytes(-1) == 128 * 128 * 2
    sp = op.space()
    assert sp.family == B.FAM_GEMM_MFMA and [sp.slots[i].name for i in range(sp.n_slots)][-1] == b"compute_at"
    t = B.trace_sample_valid(op, sp, 3, 0)
    p = B.trace_validate(op, sp, t)
    assert "op=conv1d_nwc" in B.trace_to_text(op, sp, t)
    # not the same kernel as the 1 x 3 conv2d over an image of height 1, which is also padded vertically (3 output rows)
    op2 = B.conv2d_op(1, 1, 256, 64, 128, 1, 3, stride=2, pad=1)
    assert op2.loops()[0] == ("i", 2 * 128, False)
    with pytest.raises(B.MsError):
        B.conv1d_op(1, 2, 8, 16, 5, stride=1, pad=0)                                      # empty output


def test_conv3d_descriptor_and_space():
    op = B.conv3d_op(1, 16, 224, 224, 3, 64, 7, stride=2, pad=3)
    assert op.loops() == [("i", 8 * 112 * 112, False), ("j", 64, False), ("k", 343 * 3, True)]
    assert op.desc().kind == B.OP_CONV3D_NDHWC and list(op.desc().dims)[:7] == [1, 16, 224, 224, 3, 64, 7]
    assert op.tensor_bytes(0) == 16 * 224 * 224 * 3 * 2 and op.tensor_bytes(1) == 1029 * 64 * 2
    sp = op.space()
    ca = [sp.slots[i] for i in range(sp.n_slots) if sp.slots[i].name == b"compute_at"][0]
    assert list(ca.weight)[:5] == [1, 0, 0, 0, 0]
    op2 = B.conv3d_op(2, 6, 8, 8, 16, 32, 3, stride=1, pad=1)
    sp2 = op2.space()
    t = B.trace_sample_valid(op2, sp2, 5, 0)
    p = B.trace_validate(op2, sp2, t)
    cov = B.variant_coverage(op2, p, 2 * 6 * 8 * 8 * 32)
    assert cov.min() == 1 and cov.max() == 1 and "op=conv3d_ndhwc" in B.trace_to_text(op2, sp2, t)
    # another depth is another kernel
    op3 = B.conv3d_op(2, 5, 8, 8, 16, 32, 3, stride=1, pad=1)
    assert B.trace_validate(op3, op3.space(), B.trace_sample_valid(op3, op3.space(), 5, 0)).key != p.key


def test_filter_row_layout_space_and_rules():
    op = B.conv2d_op(1, 224, 224, 3, 64, 7, 7, stride=2, pad=3)
    sp = op.space(B.SPACE_DEFAULT | B.SPACE_TAP_ROWS)
    assert sp.flags & B.SPACE_TAP_ROWS
    ks = [sp.slots[i] for i in range(sp.n_slots) if sp.slots[i].name == b"k"][0]
    tz = sp.slots[0]
    # 7 runs of 21 elements, each rounded up to the intrinsic's k: 7*32/16, 7*24/8, 7*32/32, 7*32/16
    assert {tz.candidates[c]: ks.extent_by_choice[c] for c in range(tz.n_candidates)} == {161616: 14, 323208: 21, 161632: 7, 323216: 14}
    ca = [sp.slots[i] for i in range(sp.n_slots) if sp.slots[i].name == b"compute_at"][0]
    assert list(ca.weight)[:5] == [1, 1, 1, 1, 1]
    seen = set()
    for idx in range(40):
        t = B.trace_sample_valid(op, sp, 11, idx)
        p = B.trace_validate(op, sp, t)
        assert p.tap_rows == 1 and p.tile_unit[2] * p.tk[0] * p.tk[1] * p.tk[2] * p.tk[3] in (224, 168)
        seen.add(p.compute_at)
        assert "op=conv2d_nhwc" in B.trace_to_text(op, sp, t)
    assert {0, 1, 2} <= seen
    # the same trace in the default space is another kernel (or invalid): the layout is part of the key
    assert not (op.space().flags & B.SPACE_TAP_ROWS)
    # pixels that start at odd multiples of 2 bytes: im2col staging only
    op2 = B.conv2d_op(1, 16, 16, 3, 32, 3, 3, stride=1, pad=1)
    sp2 = op2.space(B.SPACE_DEFAULT | B.SPACE_TAP_ROWS)
    ca2 = [sp2.slots[i] for i in range(sp2.n_slots) if sp2.slots[i].name == b"compute_at"][0]
    assert list(ca2.weight)[:5] == [1, 0, 0, 0, 0]
    # the flag is dropped where the layout does not apply: dilated, grouped, transposed, other operators
    assert not (B.conv2d_op(1, 16, 16, 4, 32, 3, 3, pad=2, dilation=2).space(0x2ff).flags & B.SPACE_TAP_ROWS)
    assert not (B.conv2d_op(1, 16, 16, 8, 32, 3, 3, pad=1, groups=2).space(0x2ff).flags & B.SPACE_TAP_ROWS)
    assert not (B.gemm_op(128, 128, 128, "f16").space(0x2ff).flags & B.SPACE_TAP_ROWS)


# ---------------------------------------------------------------- kernel identity

@pytest.mark.parametrize("mk", CONFIG_OPS + [lambda: B.softmax_op(1, 64, 256)])
def test_equal_kernel_text_means_equal_key(mk):
    """The key names the kernel: traces whose decisions resolve to the same template options (e.g. unroll budgets
    that are clamped alike) share one key, so a search never compiles or measures one kernel twice; different
    options give different keys."""
    op = mk()
    sp = op.space()
    by_text, by_key = {}, {}
    for idx in range(300):
        p = B.trace_validate(op, sp, B.trace_sample_valid(op, sp, 33, idx))
        text = B.variant_kernel_text(op, p)
        assert by_text.setdefault(text, p.key) == p.key, "one kernel, two keys:\n" + text
        assert by_key.setdefault(p.key, text) == text, "one key, two kernels"
    assert len(by_text) > 20


def test_unroll_budgets_that_resolve_alike_share_a_key():
    op = B.dwconv2d_op(1, 28, 28, 12)
    sp = op.space()
    t = B.trace_sample_valid(op, sp, 1, 0)
    pos = [i for i in range(sp.n_slots) if sp.slots[i].slot_id == B.SLOT_UNROLL][0]
    keys = []
    for choice in range(3):  # budgets 0, 16, 64
        t.d[pos].v[0] = choice
        keys.append(B.trace_validate(op, sp, t).key)
    assert keys[1] == keys[2] and keys[0] != keys[1]  # 16 and 64 both unroll the 9 taps fully


# ---------------------------------------------------------------- rfactor (reduction split across workgroups)

def test_rfactor_is_an_opt_in_module_with_rules():
    op = B.gemm_op(256, 256, 512, "f16")
    assert B.SLOT_RFACTOR not in [op.space().slots[i].slot_id for i in range(op.space().n_slots)]
    sp = op.space(B.SPACE_DEFAULT | B.SPACE_RFACTOR)
    s = sp.slots[sp.n_slots - 1]
    assert s.slot_id == B.SLOT_RFACTOR and [s.candidates[c] for c in range(s.n_candidates)] == [1, 2, 4, 8]
    # the vector-ALU family has no such decision
    sp_alu = B.gemm_op(128, 128, 128, "f32").space(B.SPACE_DEFAULT | B.SPACE_RFACTOR)
    assert B.SLOT_RFACTOR not in [sp_alu.slots[i].slot_id for i in range(sp_alu.n_slots)]

    def mk(k, cache=2, pad=0, reorder=0, cw=0, rf=1):
        return B.make_trace(sp, [[161632], [4, 2, 2, 1], [4, 2, 2, 1], k, [0], [cache], [8], [8], [pad], [reorder], [cw], [rf]])

    base = B.trace_validate(op, sp, mk([8, 1, 1, 2]))
    assert base.rfactor == 1 and base.grid[0] == 16
    p = B.trace_validate(op, sp, mk([8, 1, 1, 2], rf=4))
    assert p.rfactor == 4 and p.grid[0] == 64 and p.key != base.key
    assert "-DRFACTOR=4" in B.variant_kernel_text(op, p)
    assert "rfactor(loop=k0, factor=4)" in B.trace_to_text(op, sp, mk([8, 1, 1, 2], rf=4))
    for bad, why in [(mk([4, 2, 1, 2], rf=8), "does not divide"), (mk([8, 1, 1, 2], rf=2, cw=1), "cache_write"),
                     (mk([8, 1, 1, 2], cache=5, reorder=3, rf=2), "persistent")]:
        with pytest.raises(B.MsError, match=why):
            B.trace_validate(op, sp, bad)
    # launching without the workspace is refused before anything touches a device
    v = B.Variant(op, sp, mk([8, 1, 1, 2], rf=4))
    assert v.workspace_bytes() == 4 * 256 * 256 * 4
    with pytest.raises(B.MsError, match="workspace"):
        v.launch([8, 8], 8)
    with pytest.raises(B.MsError, match="aligned"):
        v.launch([8, 8], 8, workspace=4)


@pytest.mark.parametrize("mk", CONFIG_OPS + [lambda: B.softmax_op(1, 64, 256), lambda: B.norm_op(2, 32, 48),
                                             lambda: B.conv2d_op(1, 32, 32, 3, 32, 7, 7, stride=2, pad=3)])
def test_interpreter_visits_every_reduction_position_once(mk):
    """The k split (rfactor run, k0, k1, k2, k3, intrinsic k) of any valid trace visits each position of the
    reduction exactly once: nothing is dropped or counted twice, whatever the decisions."""
    op = mk()
    flags = B.SPACE_DEFAULT | B.SPACE_RFACTOR
    sp = op.space(flags)
    K = [e for n, e, red in op.loops() if red]
    for idx in range(40):
        t = B.trace_sample_valid(op, sp, 22, idx)
        p = B.trace_validate(op, sp, t)
        cov = B.variant_reduction_coverage(op, p)
        assert cov.min() == 1 and cov.max() == 1, t.decisions()
        total = int(np.prod(K))
        assert total <= len(cov) < total + max(1, p.tile_unit[2])  # a convolution may pad K up to the intrinsic's k


# ---------------------------------------------------------------- modules as data, Compose, Stochastic-Compose (Section 3.2)

def test_module_table_and_compose():
    mods = B.modules()
    names = [m["name"] for m in mods]
    assert names[0] == "multi-level-tiling" and mods[0]["flag"] == 0
    assert {"use-mfma", "cache-read", "vectorize", "unroll", "storage-align", "reorder-grid", "cache-write", "compute-location",
            "rfactor"} <= set(names)
    flags = [m["flag"] for m in mods[1:]]
    assert len(set(flags)) == len(flags) and all(f and not (f & (f - 1)) for f in flags)   # one bit each
    by_flag = {m["flag"]: m for m in mods}
    for m in mods:                                                                         # requirements name real modules
        r = m["requires"]
        while r:
            bit = r & -r
            assert bit in by_flag
            r ^= bit
    op = B.gemm_op(256, 256, 256, "f16")
    default = ["multi-level-tiling", "use-mfma", "cache-read", "vectorize", "unroll", "storage-align", "reorder-grid", "cache-write"]
    sp, mask = B.space_compose(op, default)
    assert mask == 0x7F and bytes(sp) == bytes(op.space())          # compute-location does not apply to a matrix product
    # the order of the list does not change the space (slot order is canonical), as long as requirements come first
    sp2, _ = B.space_compose(op, ["multi-level-tiling", "unroll", "use-mfma", "cache-write", "reorder-grid", "storage-align", "vectorize", "cache-read"])
    assert bytes(sp2) == bytes(sp)
    # every prefix of a list is a space of its own: the space grows module by module
    sizes = []
    for n in range(1, len(default) + 1):
        spn, maskn = B.space_compose(op, default[:n])
        sizes.append(B.space_log10_size(spn))
        assert spn.n_slots >= 3
    assert all(b >= a for a, b in zip(sizes[1:], sizes[2:]))        # (the matrix-core module changes the tile units, so [0] -> [1] may shrink)
    with pytest.raises(B.MsError, match="must start with multi-level-tiling"):
        B.space_compose(op, ["use-mfma"])
    with pytest.raises(B.MsError, match="cache-write needs use-mfma"):
        B.space_compose(op, ["multi-level-tiling", "cache-write", "use-mfma"])
    with pytest.raises(B.MsError, match="listed twice"):
        B.space_compose(op, ["multi-level-tiling", "unroll", "unroll"])
    # a module that does not apply to the operator is the identity
    dw = B.dwconv2d_op(1, 28, 28, 16)
    spd, maskd = B.space_compose(dw, default)
    assert bytes(spd) == bytes(dw.space()) and not (maskd & B.SPACE_TENSORIZE)
    conv = B.conv2d_op(1, 28, 28, 16, 32, 3, 3, stride=1, pad=1)
    spc, maskc = B.space_compose(conv, default + ["compute-location"])
    assert maskc == 0xFF and bytes(spc) == bytes(conv.space())


def test_stochastic_compose_is_seeded_and_respects_requirements():
    mods = B.modules()
    req = {m["name"]: m["requires"] for m in mods}
    flag = {m["name"]: m["flag"] for m in mods}
    op = B.conv2d_op(1, 28, 28, 16, 32, 3, 3, stride=1, pad=1)
    every = [m["name"] for m in mods]
    seen_masks, count = set(), {n: 0 for n in every}
    N = 300
    for seed in range(N):
        sp, applied = B.space_stochastic_compose(op, every, seed)
        again_sp, again = B.space_stochastic_compose(op, every, seed)
        assert applied == again and bytes(sp) == bytes(again_sp)
        assert applied[0] == "multi-level-tiling" and len(set(applied)) == len(applied)
        have = 0
        for n in applied:
            assert (req[n] & have) == req[n], (applied, n)          # requirements were applied earlier
            have |= flag[n]
            count[n] += 1
        assert sp.flags == have
        seen_masks.add(sp.flags)
        # the composed space is a working space: a valid trace can be drawn unless the conv has no vector kernel family
        if sp.flags & B.SPACE_TENSORIZE:
            B.trace_sample_valid(op, sp, 1, 0)
    assert len(seen_masks) > 30
    # the first draw at a location with c candidates applies each of them with probability 1 / (c + 1)
    assert count["use-mfma"] == N and count["use-mfma-f32"] == 0 and 0.2 * N < count["compute-location"] < 0.8 * N
    gemm = B.gemm_op(128, 128, 128, "f16")               # has a vector-ALU family: the matrix-core module is one of the draws
    n_mfma = sum("use-mfma" in B.space_stochastic_compose(gemm, every, seed)[1] for seed in range(N))
    assert 0.3 * N < n_mfma < 0.9 * N
    with pytest.raises(B.MsError, match="needs use-mfma"):
        B.space_stochastic_compose(op, ["unroll", "cache-read"], 0)
    # a restricted module set restricts the space
    sp, applied = B.space_stochastic_compose(op, ["use-mfma", "unroll"], 4)
    assert set(applied) <= {"multi-level-tiling", "use-mfma", "unroll"}
    sp, applied = B.space_stochastic_compose(B.gemm_op(128, 128, 128, "f32"), [], 0)
    assert applied == ["multi-level-tiling"] and sp.flags == 0


def test_row_major_b_layout_is_offered_and_validated():
    """storage_align 3 (B row-major in LDS, transposing LDS loads): offered for matrix-core GEMMs whose B is contiguous
    along j; the validator wants 16-byte fragments, 16-byte loads of B and register staging, and counts a dense B tile."""
    def align_candidates(op):
        sp = op.space()
        for i in range(sp.n_slots):
            if sp.slots[i].slot_id == B.SLOT_STORAGE_ALIGN:
                return [sp.slots[i].candidates[c] for c in range(sp.slots[i].n_candidates)]
        return None

    assert align_candidates(B.gemm_op(512, 512, 512, "i8")) == [0, 1, 2, 3, 4]
    assert align_candidates(B.gemm_op(1024, 1024, 1024, "f16")) == [0, 1, 2, 3, 4]
    assert align_candidates(B.bmm_op(4, 64, 64, 64, False, "f16")) == [0, 1, 2, 3, 4]
    assert align_candidates(B.bmm_op(4, 64, 64, 64, True, "f16")) == [0, 1, 2]           # B contiguous along k
    assert align_candidates(B.conv2d_op(1, 56, 56, 64, 64, 3, 3, stride=1, pad=1)) == [0, 1, 2]
    assert align_candidates(B.gemm_op(256, 256, 256, "f8", "f16")) == [0, 1, 2, 3, 4]
    assert align_candidates(B.gemm_op(128, 128, 128, "f32")) == [0, 1]                   # vector-ALU space
    op = B.gemm_op(512, 512, 512, "i8")
    sp = op.space()

    def mk(mfma=161664, k=(4, 1, 2, 1), cache=1, vec_b=16):
        return B.make_trace(sp, [[mfma], [4, 8, 1, 1], [4, 2, 4, 1], list(k), [0], [cache], [16], [vec_b], [3], [2], [0]])

    p = B.trace_validate(op, sp, mk())
    assert p.lds_pad == 3
    # A: 8 planes of 128 fragments of 16 bytes + 16 bytes of padding each; B: 128 k-rows of 128 bytes, dense
    assert p.lds_bytes == 8 * (128 * 16 + 16) + 128 * 128
    assert "transform-layout(buffer=B.lds" in B.trace_to_text(op, sp, mk())
    # 4: no swizzle, every k-row of B padded by 32 bytes
    t4 = B.make_trace(sp, [[161664], [4, 8, 1, 1], [4, 2, 4, 1], [4, 1, 2, 1], [0], [1], [16], [16], [4], [2], [0]])
    p4 = B.trace_validate(op, sp, t4)
    assert p4.lds_pad == 4 and p4.lds_bytes == 8 * (128 * 16 + 16) + 128 * (128 + 32) and p4.key != p.key
    assert "padded by 32 bytes" in B.trace_to_text(op, sp, t4)
    assert B.trace_validate(op, sp, mk(cache=2)).lds_bytes == 2 * p.lds_bytes
    assert B.trace_validate(op, sp, mk(mfma=161632, k=(4, 1, 2, 2))).lds_bytes == 16 * (128 * 8 + 16) + 128 * 128   # 8-byte fragments
    for bad, why in ((mk(vec_b=4), "vectorize_b"), (mk(cache=5), "")):
        with pytest.raises(B.MsError) as e:
            B.trace_validate(op, sp, bad)
        assert why in str(e.value)
    # a different layout is a different kernel
    q = B.trace_validate(op, sp, B.make_trace(sp, [[161664], [4, 8, 1, 1], [4, 2, 4, 1], [4, 1, 2, 1], [0], [1], [16], [16], [2], [2], [0]]))
    assert q.key != p.key and B.variant_kernel_text(op, q) != B.variant_kernel_text(op, p)
