"""Host-side checks of the C boundary that need no GPU: the library loads, exports every
function the header declares, sizes and binds layouts, and rejects bad arguments before
launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fusco.h")              # the shuffle's boundary and its variants
PROBE_HEADER = os.path.join(ROOT, "include", "fusco_probe.h")  # measurement aids of the same library


@pytest.fixture(scope="module")
def lib():
    from paper_2512_22036_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2512_22036_amd.build import build_library
        build_library()
    return binding.load_library()


def _declared_functions():
    names = set()
    for header in (HEADER, PROBE_HEADER):
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names |= set(re.findall(r"\b(fusco_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_functions_are_exported(lib):
    from paper_2512_22036_amd import binding
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_header_is_plain_c_and_cxx():
    """The boundary is a C header: it must compile on its own as C99 and as C++ (no HIP or torch types)."""
    import shutil
    import subprocess
    if not shutil.which("gcc") or not shutil.which("g++"):
        pytest.skip("no host compiler")
    for header in (HEADER, PROBE_HEADER):
        subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", header])
        subprocess.check_call(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", header])
        text = open(header).read()
        assert "hip/" not in text and "torch" not in text.lower()
    assert "probe" not in open(HEADER).read().lower()      # the aids stay out of the shuffle's header


def test_version_and_status_strings(lib):
    assert lib.fusco_version() == 110
    assert lib.fusco_status_string(0) == b"ok"
    for code in (-1, -2, -3, -4, -99):
        assert len(lib.fusco_status_string(code)) > 0


def test_layout_sizes(lib):
    assert lib.fusco_layout_bytes(8192, 8, 256, 8) >= 4 * (7 * 65536 + 2 * 257 + 2 * 9) + 65536
    assert lib.fusco_layout_bytes(0, 8, 256, 8) > 0
    assert lib.fusco_scratch_bytes(8192, 8, 256, 8) >= 32 * (256 + 8 + 1) * 4
    bad = [(-1, 8, 256, 8), (16, 0, 256, 8), (16, 65, 256, 8), (16, 8, 0, 8), (16, 8, 2048, 8),
           (16, 8, 256, 0), (16, 8, 256, 3), (16, 8, 8, 16), (1 << 30, 8, 256, 8)]
    for args in bad:
        assert lib.fusco_layout_bytes(*args) == 0, args
        assert lib.fusco_scratch_bytes(*args) == 0, args


def test_layout_bind_carves_disjoint_aligned_arrays(lib):
    from paper_2512_22036_amd.binding import _CLayout
    N, k, E, D = 100, 4, 16, 8
    nbytes = lib.fusco_layout_bytes(N, k, E, D)
    base = 0x10000000   # never dereferenced: bind is host-only pointer arithmetic
    L = _CLayout()
    assert lib.fusco_layout_bind(ctypes.byref(L), N, k, E, D, base, nbytes) == 0
    assert (L.N, L.k, L.E, L.D, L.P, L.send_cap) == (N, k, E, D, N * k, N * min(k, D))
    sizes = dict(exp_count=4 * E, exp_off=4 * (E + 1), send_count=4 * D, send_off=4 * (D + 1), pair_slot=4 * N * k,
                 slot_pair=4 * N * k, slot_token=4 * N * k, send_src=4 * L.send_cap, pair_send_row=4 * N * k,
                 slot_send_row=4 * N * k, pair_first=N * k, status=4,
                 tile_slots=4 * L.tile_count * L.tile_tokens * k)
    assert (L.tile_tokens, L.tile_count) == (1024 // k, 1)          # 400 pairs: a single tile of one round
    L2 = _CLayout()
    assert lib.fusco_layout_bind(ctypes.byref(L2), 8192, 8, 256, 8, base, lib.fusco_layout_bytes(8192, 8, 256, 8)) == 0
    assert (L2.tile_tokens, L2.tile_count) == (256, 32)            # tiles of 2048 pairs
    spans = sorted((getattr(L, n), getattr(L, n) + s) for n, s in sizes.items())
    assert spans[0][0] >= base and spans[-1][1] <= base + nbytes
    for (a0, a1), (b0, _) in zip(spans, spans[1:]):
        assert a1 <= b0
    assert all(a0 % 256 == 0 for a0, _ in spans)
    assert lib.fusco_layout_bind(ctypes.byref(L), N, k, E, D, base, nbytes - 1) == -2
    assert lib.fusco_layout_bind(ctypes.byref(L), N, k, E, D, base + 16, nbytes) == -1
    assert lib.fusco_layout_bind(ctypes.byref(L), N, k, E, D, None, nbytes) == -1
    assert lib.fusco_layout_bind(None, N, k, E, D, base, nbytes) == -1
    assert lib.fusco_layout_bind(ctypes.byref(L), N, k, E, 5, base, nbytes) == -1


def test_entry_points_reject_bad_arguments_without_launching(lib):
    from paper_2512_22036_amd.binding import _CLayout
    N, k, E, D = 64, 2, 8, 4
    nbytes = lib.fusco_layout_bytes(N, k, E, D)
    base, buf = 0x10000000, 0x20000000
    L = _CLayout()
    assert lib.fusco_layout_bind(ctypes.byref(L), N, k, E, D, base, nbytes) == 0
    scratch = lib.fusco_scratch_bytes(N, k, E, D)
    # plan
    assert lib.fusco_plan(ctypes.byref(L), None, buf, scratch, None) == -1
    assert lib.fusco_plan(ctypes.byref(L), buf, None, scratch, None) == -1
    assert lib.fusco_plan(ctypes.byref(L), buf, buf, scratch - 1, None) == -2
    assert lib.fusco_plan(None, buf, buf, scratch, None) == -1
    empty = _CLayout()
    assert lib.fusco_plan(ctypes.byref(empty), buf, buf, scratch, None) == -1
    # plan on the library's static scratch: same checks, plus its size limit (refused before any device call)
    assert lib.fusco_plan_static(ctypes.byref(L), None, None) == -1
    assert lib.fusco_plan_static(None, buf, None) == -1
    assert lib.fusco_plan_static(ctypes.byref(empty), buf, None) == -1
    Lhuge = _CLayout()
    huge = (1000000, 8, 256, 8)
    assert lib.fusco_scratch_bytes(*huge) > (4 << 20) >= lib.fusco_scratch_bytes(990000, 8, 256, 8)
    assert lib.fusco_layout_bind(ctypes.byref(Lhuge), *huge, base + (1 << 27), lib.fusco_layout_bytes(*huge)) == 0
    assert lib.fusco_plan_static(ctypes.byref(Lhuge), buf, None) == -5
    assert b"static" in lib.fusco_status_string(-5)
    # dispatch
    d = lambda *a: lib.fusco_dispatch(ctypes.byref(L), *a)
    assert d(None, 64, None, 0, buf, None, None, None, 0, None) == -1            # no x
    assert d(buf, 0, None, 0, buf, None, None, None, 0, None) == -1              # empty rows
    assert d(buf, 40, None, 0, buf, None, None, None, 0, None) == -1             # not a multiple of 16
    assert d(buf, 64, None, 8, buf, None, None, None, 0, None) == -1             # aux not a multiple of 16
    assert d(buf, 64, None, 16, buf, buf, None, None, 0, None) == -1             # aux plane without source
    assert d(buf, 64, buf, 16, buf, None, None, None, 0, None) == -1             # aux plane without target
    assert d(buf, 64, None, 0, None, None, None, None, 0, None) == -1            # no expert buffer
    assert d(buf, 64, None, 0, buf, None, None, None, 2, None) == -1             # wire without send buffer
    assert d(buf + 4, 64, None, 0, buf, None, None, None, 0, None) == -1         # misaligned
    assert d(buf, 64, None, 0, buf, None, None, None, 16, None) == -3            # unknown flag
    assert d(buf, 64, None, 0, buf, None, buf, None, 4 | 8, None) == -3          # two-hop cannot stream its first hop
    assert d(buf, 64, None, 0, None, None, None, None, 8, None) == -1            # streaming alone still means the expert tensor
    assert d(buf, 64, None, 0, buf, None, None, None, 4, None) == -1             # two-hop needs the send buffer
    assert d(buf, 16 << 20, None, 0, buf, None, None, None, 0, None) == -1       # row too large
    assert d(buf, (1 << 20) + 16, None, 0, buf, None, None, None, 0, None) == -1 # just above FUSCO_MAX_ROW_BYTES
    assert d(buf, 1 << 20, buf, 16, buf, buf, None, None, 0, None) == -1         # the two planes together are
    # fused plan + dispatch
    pd = lambda *a: lib.fusco_plan_dispatch(ctypes.byref(L), *a)
    assert pd(None, buf, 64, None, 0, buf, None, None) == -1                     # no routing
    assert pd(buf, None, 64, None, 0, buf, None, None) == -1                     # no x
    assert pd(buf, buf, 64, None, 0, None, None, None) == -1                     # no expert tensor
    assert pd(buf, buf, 40, None, 0, buf, None, None) == -1                      # row size
    assert pd(buf, buf, 64, None, 16, buf, None, None) == -1                     # aux plane without tensors
    assert pd(buf, buf + 8, 64, None, 0, buf, None, None) == -1                  # misaligned
    Lbig = _CLayout()
    assert lib.fusco_layout_bind(ctypes.byref(Lbig), 2049, 1, E, D, base + (1 << 26), lib.fusco_layout_bytes(2049, 1, E, D)) == 0
    assert lib.fusco_plan_dispatch(ctypes.byref(Lbig), buf, buf, 64, None, 0, buf, None, None) == -3   # more than one tile
    # an empty layout takes NULL tensors (nothing is launched), sizes are still checked
    L0 = _CLayout()
    assert lib.fusco_layout_bind(ctypes.byref(L0), 0, k, E, D, base + (1 << 25), lib.fusco_layout_bytes(0, k, E, D)) == 0
    assert lib.fusco_dispatch(ctypes.byref(L0), None, 64, None, 0, None, None, None, None, 3, None) == 0
    assert lib.fusco_dispatch(ctypes.byref(L0), None, 40, None, 0, None, None, None, None, 0, None) == -1
    assert lib.fusco_combine(ctypes.byref(L0), None, 0, None, None, 0, 64, 0, None) == 0
    assert lib.fusco_combine(ctypes.byref(L0), None, 0, None, None, 0, 12, 0, None) == -1
    assert lib.fusco_combine(ctypes.byref(L0), None, 5, None, None, 0, 64, 0, None) == -3
    assert lib.fusco_combine_two_hop(ctypes.byref(L0), None, 0, None, None, None, 0, 64, None) == 0
    # combine
    c = lambda *a: lib.fusco_combine(ctypes.byref(L), *a)
    assert c(None, 0, buf, buf, 0, 64, 0, None) == -1
    assert c(buf, 0, None, buf, 0, 64, 0, None) == -1
    assert c(buf, 0, buf, None, 0, 64, 0, None) == -1
    assert c(buf, 0, buf, buf, 0, 0, 0, None) == -1
    assert c(buf, 0, buf, buf, 0, 12, 0, None) == -1          # 24-byte rows
    assert c(buf, 1, buf, buf, 1, 6, 0, None) == -1
    assert c(buf, 2, buf, buf, 0, 64, 0, None) == -3          # unknown dtype
    assert c(buf, 0, buf, buf, 7, 64, 0, None) == -3
    assert c(buf, 0, buf, buf, 0, 64, 1, None) == -3          # flags must be 0
    assert c(buf + 8, 0, buf, buf, 0, 64, 0, None) == -1
    assert c(buf, 0, buf, buf, 0, (1 << 19) + 8, 0, None) == -1   # bf16 row above FUSCO_MAX_ROW_BYTES
    assert c(buf, 1, buf, buf, 0, (1 << 18) + 4, 0, None) == -1   # fp32 row above it
    # two-hop combine
    th = lambda *a: lib.fusco_combine_two_hop(ctypes.byref(L), *a)
    assert th(buf, 0, buf, None, buf, 0, 64, None) == -1          # no partial tensor
    assert th(buf, 0, buf, buf + 4, buf, 0, 64, None) == -1       # misaligned partial tensor
    assert th(None, 0, buf, buf, buf, 0, 64, None) == -1
    assert th(buf, 0, buf, buf, buf, 5, 64, None) == -3
    assert th(buf, 0, buf, buf, buf, 0, 20, None) == -1
    # segment engine
    assert lib.fusco_segments_scan(None, 4, buf, buf, None) == -1
    assert lib.fusco_segments_scan(buf, -1, buf, buf, None) == -1
    assert lib.fusco_segments_scan(buf, 4, None, buf, None) == -1
    assert lib.fusco_segments_scan(buf, 4, buf, None, None) == -1
    assert lib.fusco_segments_scan(buf, 1 << 27, buf, buf, None) == -1
    sc = lambda *a: lib.fusco_segments_copy(*a)
    assert sc(None, 64, buf, buf, 64, None, buf, 1, 64, 0, None, buf, None) == -1
    assert sc(buf, 64, buf, None, 64, None, buf, 1, 64, 0, None, buf, None) == -1
    assert sc(buf, 64, buf, buf, 64, None, None, 1, 64, 0, None, buf, None) == -1
    assert sc(buf, 64, buf, buf, 64, None, buf, 1, 64, 0, None, None, None) == -1
    assert sc(buf + 8, 64, buf, buf, 64, None, buf, 1, 64, 0, None, buf, None) == -1
    assert sc(buf, 64, buf, buf, 64, None, buf, 1, 64, 1000, buf, buf, None) == -1      # slice size not a multiple of 16384
    assert sc(buf, 64, buf, buf, 64, None, buf, 1, 64, 0, buf, buf, None) == -1         # slice counters without a slice size
    # disaggregated baseline
    Lr = _CLayout()
    assert lib.fusco_layout_bind(ctypes.byref(Lr), N, k, D, D, base + (1 << 24), lib.fusco_layout_bytes(N, k, D, D)) == 0
    rscratch = lib.fusco_scratch_bytes(N, k, D, D)
    assert lib.fusco_disaggregated_plan(ctypes.byref(Lr), ctypes.byref(L), None, buf, buf, rscratch, None) == -1
    assert lib.fusco_disaggregated_plan(ctypes.byref(Lr), ctypes.byref(L), buf, None, buf, rscratch, None) == -1
    assert lib.fusco_disaggregated_plan(ctypes.byref(L), ctypes.byref(L), buf, buf, buf, rscratch, None) == -1   # not (N,k,D,D)
    assert lib.fusco_disaggregated_plan(ctypes.byref(Lr), ctypes.byref(L), buf, buf, buf, rscratch - 1, None) == -2
    dd = lambda *a: lib.fusco_disaggregated_dispatch(ctypes.byref(L), ctypes.byref(Lr), *a)
    assert dd(None, 64, buf, buf, buf, None) == -1
    assert dd(buf, 40, buf, buf, buf, None) == -1
    assert dd(buf, 64, None, buf, buf, None) == -1
    assert dd(buf, 64, buf, buf + 8, buf, None) == -1
    assert lib.fusco_disaggregated_dispatch(ctypes.byref(L), ctypes.byref(L), buf, 64, buf, buf, buf, None) == -1
    dc = lambda *a: lib.fusco_disaggregated_combine(ctypes.byref(L), ctypes.byref(Lr), *a)
    assert dc(buf, 0, buf, None, buf, buf, 0, 64, None) == -1
    assert dc(buf, 0, buf, buf, buf, None, 0, 64, None) == -1
    assert dc(buf, 3, buf, buf, buf, buf, 0, 64, None) == -3
    assert dc(buf, 0, buf, buf, buf, buf, 0, 12, None) == -1
    assert lib.fusco_disaggregated_plan(ctypes.byref(Lr), ctypes.byref(L), buf, buf, None, rscratch, None) == -1  # no scratch
    # cross-node load of the balancer
    cl = lambda *a: lib.fusco_cross_node_load(ctypes.byref(L), *a)
    assert cl(2, 0, 64, None, None) == -1                     # no result cell
    assert cl(2, 0, 64, buf + 4, None) == -1                  # misaligned cell
    assert cl(3, 0, 64, buf, None) == -1                      # D = 4 is not a multiple of 3
    assert cl(0, 0, 64, buf, None) == -1
    assert cl(2, 2, 64, buf, None) == -1                      # only nodes 0 and 1 exist
    assert cl(2, -1, 64, buf, None) == -1
    assert cl(2, 0, 0, buf, None) == -1
    assert lib.fusco_cross_node_load(None, 2, 0, 64, buf, None) == -1
    # probe copy
    assert lib.fusco_probe_copy(None, buf, 64, None) == -1
    assert lib.fusco_probe_copy(buf, buf + 4, 64, None) == -1
    assert lib.fusco_probe_copy(buf, buf + 4096, 24, None) == -1
    assert lib.fusco_probe_copy(buf, buf + 4096, 0, None) == 0
    assert lib.fusco_probe_time_next_call(None, buf) == -1 and lib.fusco_probe_time_next_call(buf, None) == -1
    # probe pieces
    lib.fusco_probe_source_chunk_bytes.restype = ctypes.c_size_t
    lib.fusco_probe_source_chunk_bytes.argtypes = [ctypes.c_size_t]
    assert lib.fusco_probe_source_chunk_bytes(0) == 128 << 20              # reading leaves the value alone
    assert lib.fusco_probe_source_chunk_bytes(1 << 20) == 128 << 20 and lib.fusco_probe_source_chunk_bytes(0) == 1 << 20
    assert lib.fusco_probe_source_chunk_bytes(128 << 20) == 1 << 20
    assert lib.fusco_probe_dispatch_kernel(-1) == 0 and lib.fusco_probe_dispatch_kernel(1) == 0
    assert lib.fusco_probe_dispatch_kernel(-1) == 1 and lib.fusco_probe_dispatch_kernel(0) == 1
    assert lib.fusco_probe_dispatch_kernel(2) == 0 and lib.fusco_probe_dispatch_kernel(0) == 2
    assert lib.fusco_probe_dispatch_kernel(3) == -1 and lib.fusco_probe_dispatch_kernel(-1) == 0
    assert lib.fusco_probe_dispatch_occupancy(-1) == 0 and lib.fusco_probe_dispatch_occupancy(5) == 0
    assert lib.fusco_probe_dispatch_occupancy(-1) == 5 and lib.fusco_probe_dispatch_occupancy(16) == 5
    assert lib.fusco_probe_dispatch_occupancy(2) == -1 and lib.fusco_probe_dispatch_occupancy(17) == -1    # 1, 2 and > 16 refused
    assert lib.fusco_probe_dispatch_occupancy(0) == 16 and lib.fusco_probe_dispatch_occupancy(-1) == 0
    assert lib.fusco_probe_dispatch_walk(-1) == 0 and lib.fusco_probe_dispatch_walk(4) == 0
    assert lib.fusco_probe_dispatch_walk(5) == -1 and lib.fusco_probe_dispatch_walk(0) == 4 and lib.fusco_probe_dispatch_walk(-1) == 0
    assert lib.fusco_probe_dispatch_pull(-1) == 0 and lib.fusco_probe_dispatch_pull(2) == 0
    assert lib.fusco_probe_dispatch_pull(1) == 2 and lib.fusco_probe_dispatch_pull(3) == -1
    assert lib.fusco_probe_dispatch_pull(0) == 1 and lib.fusco_probe_dispatch_pull(-1) == 0
    pp = lib.fusco_probe_pieces
    assert pp(None, 1 << 20, 1, 1, 0, None, None) == -1
    assert pp(buf, (1 << 20) + 16, 1, 1, 0, None, None) == -1              # not whole pieces
    assert pp(buf, 4096 * 12, 1, 1, 0, None, None) == -1                   # pieces not a multiple of 8
    assert pp(buf, 4096 * 64, 1, 3, 0, None, None) == -1                   # 8 pieces per XCD do not split into runs of 3
    assert pp(buf, 4096 * 64, 1, 0, 0, None, None) == -1
    assert pp(buf, 4096 * 64, 0, 1, 0, None, None) == -1                   # reads need the sink
    assert pp(buf + 8, 4096 * 64, 1, 1, 0, None, None) == -1
    assert pp(buf, 4096 * 2, 1, 1, 1, None, None) == -1                    # too few pieces to scatter
    # probe rows: unsupported shapes, bad sizes, missing buffers (nothing is launched on error)
    pr = lib.fusco_probe_rows
    assert pr(buf, 8, buf + 4096, 8, 64, 2, 1, 0, 0, None, None) == -1        # shape not offered
    assert pr(buf, 8, buf + 4096, 8, 24, 1, 1, 0, 0, None, None) == -1        # row size not a multiple of 16
    assert pr(None, 8, buf + 4096, 8, 64, 1, 1, 0, 0, None, None) == -1
    assert pr(buf, 8, None, 8, 64, 1, 1, 0, 0, None, None) == -1
    assert pr(buf, 8, buf + 4096, 12, 64, 1, 8, 0, 0, None, None) == -1       # 12 rows do not split into groups of 8
    assert pr(buf, 1, buf + 4096, 16, 64, 1, 8, 0, 0, None, None) == -1       # 2 groups need 2 source rows
    assert pr(buf, 8, None, 0, 64, 1, 0, 0, 0, None, None) == -1              # read-only shape needs the sink
    assert pr(buf, 8, buf + 4100, 8, 64, 1, 1, 0, 0, None, None) == -1        # misaligned


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2512_22036_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "fusco_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2512_22036_amd" not in text and "libfusco.so" not in text, f
