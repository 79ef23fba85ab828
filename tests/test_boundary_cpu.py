"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes payloads as the paper's accounting implies, and rejects bad arguments
before launching anything."""
import ctypes as C
import os
import re

import pytest

import paper_2506_21263_amd as dlcx

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dlcx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dlcx_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = C.CDLL(dlcx.LIB_PATH)
    names = declared_symbols()
    assert {"dlcx_delta_ef", "dlcx_compress", "dlcx_average", "dlcx_decompress",
            "dlcx_outer_nesterov", "dlcx_select_rank"} <= set(names)
    for name in names:
        assert hasattr(L, name), name
    assert set(names) == set(dlcx.SYMBOLS), set(names) ^ set(dlcx.SYMBOLS)


def test_payload_bytes_follow_the_layout():
    d = dlcx.desc(8192, 8192, 64, 4, 128)
    total, cb, sb = dlcx.dlcx_payload_bytes(d, dlcx.PHASE_P)
    assert cb == 8192 * 64 // 2 and sb == 8192 * 64 // 128 * 4 and total == cb + sb
    d8 = dlcx.desc(512, 1024, 8, 8, 64)
    assert dlcx.dlcx_payload_bytes(d8, dlcx.PHASE_Q)[1:] == (1024 * 8, 1024 * 8 // 64 * 4)
    # config 0: (m + n) r = 8192 factor elements -> 4096 + 512 = 4608 payload bytes per worker
    d0 = dlcx.desc(512, 512, 8, 4, 64)
    assert dlcx.dlcx_payload_bytes(d0, 0)[0] + dlcx.dlcx_payload_bytes(d0, 1)[0] == 4608
    assert dlcx.dlcx_workspace_bytes(d, 4) >= 4 * 64 * 8192 * 4


@pytest.mark.parametrize("bad", [
    dict(m=0), dict(n=-16), dict(r=0), dict(r=257), dict(r=600), dict(qbits=3), dict(qbits=16),
    dict(group=48), dict(group=0), dict(m=520), dict(mma=4), dict(mma=-1)])
def test_bad_descriptors_are_rejected(bad):
    kw = dict(m=512, n=512, r=8, qbits=4, group=64, mma=0)
    kw.update(bad)
    d = dlcx.desc(**kw)
    assert dlcx.dlcx_payload_bytes(d, 0)[0] == 0
    assert dlcx.dlcx_workspace_bytes(d, 2) == 0
    L = dlcx.lib()
    fake = 0x1000  # aligned, never dereferenced: validation fails first
    assert L.dlcx_compress(C.byref(d), 0, fake, fake, fake, fake, fake, None) == dlcx.EINVAL
    assert L.dlcx_decompress(C.byref(d), fake, fake, fake, 0, None, fake, None) == dlcx.EINVAL


def test_null_misaligned_and_range_arguments():
    L = dlcx.lib()
    fake = 0x1000
    assert L.dlcx_delta_ef(None, fake, 0, fake, 16, None) == dlcx.EINVAL
    assert L.dlcx_delta_ef(fake, fake, 0, fake + 4, 16, None) == dlcx.EINVAL   # misaligned
    assert L.dlcx_delta_ef(fake, fake, 7, fake, 16, None) == dlcx.EINVAL      # dtype
    assert L.dlcx_delta_ef(fake, fake, 0, fake, -1, None) == dlcx.EINVAL
    assert L.dlcx_delta_ef(None, None, 0, None, 0, None) == dlcx.OK           # empty input
    assert L.dlcx_outer_nesterov(fake, None, fake, 4, 0.7, 0.9, None) == dlcx.EINVAL
    assert L.dlcx_outer_nesterov(None, None, None, 0, 0.7, 0.9, None) == dlcx.OK
    assert L.dlcx_quantize(fake, 100, 4, 64, fake, fake, None) == dlcx.EINVAL  # count % group
    assert L.dlcx_quantize(fake, 128, 5, 64, fake, fake, None) == dlcx.EINVAL
    assert L.dlcx_quantize(None, 0, 4, 64, None, None, None) == dlcx.OK
    d = dlcx.desc(512, 512, 8, 4, 64)
    assert L.dlcx_compress(C.byref(d), 2, fake, fake, fake, fake, fake, None) == dlcx.EINVAL
    assert L.dlcx_compress(C.byref(d), 0, fake, fake, fake, fake, None, None) == dlcx.EINVAL
    assert L.dlcx_average(C.byref(d), 0, 0, fake, fake, fake, fake, None) == dlcx.EINVAL  # K = 0
    assert L.dlcx_average(C.byref(d), 0, 17, fake, fake, fake, fake, None) == dlcx.EINVAL
    assert L.dlcx_orthonormalize(100, 4, fake, fake, None) == dlcx.EINVAL      # L % 16
    assert L.dlcx_effective_rank(64, 4, fake, 1.5, fake, fake, None) == dlcx.EINVAL  # tau
    assert dlcx.lib().dlcx_strerror(dlcx.EINVAL) == b"invalid argument"


def test_select_rank_window_rule_on_the_host(golden):
    g = golden("adagradcmp_window.txt")
    c, r1, H1 = int(g["c"][0]), int(g["r1"][0]), int(g["H1"][0])
    hist = (C.c_int32 * c)()
    for t in range(1, 9):
        rp, r, H = dlcx.dlcx_select_rank([], [], 0.99, hist, t, c, r1, 4, r1, H1,
                                         rprime=int(g["rprime"][t - 1]))
        assert (rp, r, H) == (int(g["rprime"][t - 1]), int(g["r_t"][t - 1]), int(g["H_t"][t - 1]))
    with pytest.raises(dlcx.DlcxError):
        dlcx.dlcx_select_rank([], [], 0.99, hist, 0, c, r1, 4, r1, H1, rprime=4)


def test_quantise_only_entry_points_reject_bad_arguments():
    L = dlcx.lib()
    fake = 0x1000
    arr = (C.c_void_p * 2)(fake, fake)
    ap = C.cast(arr, C.c_void_p)
    ok_args = [256, 4, 64, 2, ap, 0, ap, fake, fake, 0.7, 0.9, None, None, 0, ap, ap, None]

    def call(**kw):
        a = list(ok_args)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return L.dlcx_quant_round(*a)

    assert call(_0=100) == dlcx.EINVAL          # numel % group
    assert call(_1=5) == dlcx.EINVAL            # qbits
    assert call(_2=48) == dlcx.EINVAL           # group
    assert call(_3=0) == dlcx.EINVAL            # K
    assert call(_5=3) == dlcx.EINVAL            # dtype
    assert call(_11=ap) == dlcx.EINVAL          # previous codes without previous scales
    assert call(_7=None) == dlcx.EINVAL         # theta_g
    assert call(_11=ap, _12=ap, _8=None) == dlcx.EINVAL   # a previous payload needs v
    assert call(_0=0) == dlcx.OK                # empty tensor: nothing launched
    assert L.dlcx_requantize(fake, 100, 4, 64, None) == dlcx.EINVAL
    assert L.dlcx_requantize(fake + 4, 128, 4, 64, None) == dlcx.EINVAL
    assert L.dlcx_requantize(None, 0, 4, 64, None) == dlcx.OK
    assert L.dlcx_ef_update(2, ap, None, 64, None) == dlcx.EINVAL
    assert L.dlcx_ef_update(17, ap, fake, 64, None) == dlcx.EINVAL
    assert L.dlcx_ef_update(0, None, None, 64, None) == dlcx.OK


def test_comm_model_and_overlap_plan_on_the_host(golden):
    # the library's host-side planner against the oracle's exhaustive one (Sec. 2.4.1, 2.3)
    from oracle import planner
    g = golden("compression_accounting.txt")
    hours = dlcx.dlcx_comm_seconds(100e9 * 4, 3, 1e9) / 3600
    assert abs(hours - g["allreduce_hours"][0]) < 0.01
    assert dlcx.dlcx_comm_seconds(1e9, 0, 1e9) < 0          # bad arguments
    shapes = [(8192, 8192), (8192, 1024), (8192, 28672), (28672, 8192), (512, 256)]
    for qbits, group in ((4, 128), (8, 64)):
        descs = [dlcx.desc(m, n, 1, qbits, group) for m, n in shapes]
        for step, H, extra, iters in ((0.05, 1, 0.0, 1), (0.05, 3, 1e6, 1), (1e-3, 1, 0.0, 1),
                                      (10.0, 1, 0.0, 1), (0.05, 1, 0.0, 2), (0.05, 3, 1e6, 3)):
            want = planner.plan_overlap(shapes, qbits, group, extra, 4, 256, 3, 1e9, step, H, iters)
            got = dlcx.dlcx_plan_overlap(descs, extra, 4, 256, 3, 1e9, step, H, iters)
            assert got[:2] == want[:2]
            assert abs(got[2] - want[2]) <= 1e-12 * max(want[2], 1.0)
    with pytest.raises(dlcx.DlcxError):
        dlcx.dlcx_plan_overlap([dlcx.desc(512, 512, 1, 4, 64)], 0.0, 8, 4, 3, 1e9, 1.0, 1)
    with pytest.raises(dlcx.DlcxError):
        dlcx.dlcx_plan_overlap([dlcx.desc(512, 512, 1, 4, 64)], 0.0, 4, 8, 3, 1e9, 1.0, 1, 0)


def test_stage_lane_plan_covers_every_matrix_once_and_balances():
    # host-side scheduling of a stage: consecutive runs per stream, batches inside a run
    from paper_2506_21263_amd.stage import plan_lanes
    layer = [8192 * 8192, 8192 * 1024, 8192 * 1024, 8192 * 8192, 8192 * 28672, 8192 * 28672,
             28672 * 8192]
    cases = [(layer * 10, 3, 0), (layer * 10, 3, 4), (layer * 10, 1, 0), (layer * 5, 4, 7),
             ([5, 1, 1, 1], 3, 0), ([1], 3, 2), ([7] * 5, 2, 2)]
    for sizes, ns, chunk in cases:
        lane_of, lane_chunks = plan_lanes(sizes, ns, chunk)
        assert len(lane_of) == len(sizes) and len(lane_chunks) == ns
        assert lane_of == sorted(lane_of)                       # consecutive runs
        covered = [a for chunks in lane_chunks for lo, hi in chunks for a in range(lo, hi)]
        assert covered == list(range(len(sizes)))               # every matrix exactly once
        for lane, chunks in enumerate(lane_chunks):
            assert all(lane_of[a] == lane for lo, hi in chunks for a in range(lo, hi))
            assert all(hi > lo for lo, hi in chunks)
            assert all(c[1] == d[0] for c, d in zip(chunks, chunks[1:]))
            if chunk > 0:
                assert all(hi - lo <= chunk for lo, hi in chunks)
    lane_of, lane_chunks = plan_lanes(layer * 10, 3, 0)
    share = [sum(s for s, l in zip(layer * 10, lane_of) if l == lane) for lane in range(3)]
    assert max(share) <= 1.15 * min(share)                      # about equal element counts
    # streams out of phase: first batches of 1/3, 2/3 and all of a run
    firsts = [c[0][1] - c[0][0] for c in lane_chunks]
    runs = [c[-1][1] - c[0][0] for c in lane_chunks]
    assert firsts == [max(1, runs[l] * (l + 1) // 3) for l in range(3)]


def test_static_scratch_entry_point_limits_and_argument_errors():
    """dlcx_average_static rejects on the host, before any HIP call: bad arguments as
    dlcx_average does, and factors whose orthonormalisation scratch exceeds the fixed array."""
    L = dlcx.lib()
    cap = dlcx.dlcx_static_scratch_bytes()
    assert cap == 32 << 20
    for r, m_fits in ((256, 31232), (64, 522752)):
        fits = dlcx.desc(m_fits, 256, r, 4, 128, 2)
        over = dlcx.desc(m_fits + 512, 256, r, 4, 128, 2)
        assert 0 < dlcx.dlcx_static_scratch_need(fits, dlcx.PHASE_P) <= cap
        assert dlcx.dlcx_static_scratch_need(over, dlcx.PHASE_P) > cap
        assert dlcx.dlcx_static_scratch_need(over, dlcx.PHASE_Q) == 0
    # every shape of the benchmark configurations fits at the largest rank
    for m in (512, 2048, 8192, 28672):
        assert dlcx.dlcx_static_scratch_need(dlcx.desc(m, 1024, min(m, 256), 4, 128, 2), 0) <= cap
    fake = 0x1000
    arr = (C.c_void_p * 2)(fake, fake)
    over = dlcx.desc(65536, 256, 256, 4, 128, 2)
    ok = dlcx.desc(512, 512, 8, 4, 64, 2)
    assert L.dlcx_average_static(C.byref(over), 0, 2, arr, arr, fake, None) == dlcx.ETOOBIG
    assert L.dlcx_average_static(C.byref(ok), 0, 0, arr, arr, fake, None) == dlcx.EINVAL
    assert L.dlcx_average_static(C.byref(ok), 2, 2, arr, arr, fake, None) == dlcx.EINVAL
    assert L.dlcx_average_static(C.byref(ok), 0, 2, arr, arr, fake + 4, None) == dlcx.EINVAL
    assert L.dlcx_average_static(C.byref(ok), 0, 2, None, arr, fake, None) == dlcx.EINVAL
    bad = (C.c_void_p * 2)(fake, None)
    assert L.dlcx_average_static(C.byref(ok), 0, 2, bad, arr, fake, None) == dlcx.EINVAL
    assert L.dlcx_strerror(dlcx.ETOOBIG) == b"larger than the fixed scratch of this entry point"
