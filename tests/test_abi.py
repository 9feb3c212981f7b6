"""The C-ABI library loads, exports every function the headers under include/ declare, and exports no
signmuon_* symbol that they do not declare (no GPU needed)."""
import ctypes
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "signmuon.h")
DEBUG_HEADER = os.path.join(ROOT, "include", "signmuon_debug.h")
LIB = os.path.join(ROOT, "paper_2605_16311_amd", "libsignmuon.so")


def declared_functions(header=HEADER):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(signmuon_[a-z0-9_]+)\s*\(", text)))


def exported_symbols():
    out = subprocess.run(["nm", "-D", "--defined-only", LIB], check=True, capture_output=True, text=True).stdout
    syms = set()
    for line in out.splitlines():
        parts = line.split()
        if len(parts) >= 3 and parts[1] in "TtWw" and parts[2].startswith("signmuon_"):
            syms.add(parts[2])
    return sorted(syms)


def test_every_exported_symbol_is_declared_in_a_header():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} missing: run __graft_entry__.build() first")
    declared = set(declared_functions(HEADER)) | set(declared_functions(DEBUG_HEADER))
    exported = exported_symbols()
    assert exported, "nm found no signmuon_* symbols"
    assert set(exported) == declared, (sorted(set(exported) - declared), sorted(declared - set(exported)))


def test_header_declares_the_five_path_calls():
    names = declared_functions()
    for n in ("signmuon_momentum", "signmuon_polar_ns", "signmuon_sign_pack",
              "signmuon_majority_vote", "signmuon_step"):
        assert n in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} missing: run __graft_entry__.build() first")
    import torch  # noqa: F401  (loads the HIP runtime the library links against)
    lib = ctypes.CDLL(LIB)
    for n in declared_functions() + declared_functions(DEBUG_HEADER):
        assert hasattr(lib, n), n


def test_binding_mirrors_the_abi_and_status_text():
    from paper_2605_16311_amd import binding as B
    assert set(B.EXPORTS) == set(declared_functions())
    for n in ("signmuon_momentum", "signmuon_polar_ns", "signmuon_sign_pack",
              "signmuon_majority_vote", "signmuon_step"):
        assert callable(getattr(B, n))
    assert B._lib.signmuon_strerror(0) == b"ok"
    assert B._lib.signmuon_strerror(-1) == b"invalid argument"
    assert ctypes.sizeof(B.StepArgs) == 144  # sizeof(signmuon_step_args) under the LP64 C ABI


def test_no_gpu_means_loud_failure():
    import torch
    from paper_2605_16311_amd import binding as B
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(B.SignMuonError):
        B.Context()


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2605_16311_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src, f


def _tile_ranges(lib, probs, sym, ts):
    import ctypes as C
    n = len(probs)
    arr = lambda vals: (C.c_int * n)(*vals)
    xcd = (C.c_int * 9)()
    begin = (C.c_int * n)()
    total = lib.signmuon_debug_tile_ranges(n, arr([p[0] for p in probs]), arr([p[1] for p in probs]),
                                           arr([p[2] for p in probs]), arr([p[3] for p in probs]),
                                           arr([p[4] for p in probs]), int(sym), ts, xcd, begin)
    return total, list(xcd), list(begin)


def test_gemm_tile_ranges_cover_the_list_and_balance_cost():
    """Host logic of the grouped GEMM launch: the tile list of a launch is cut into eight contiguous
    ranges (one per XCD) of nearly equal estimated cost; a problem with a mate owns both problems' tiles."""
    import ctypes as C
    import torch  # noqa: F401  (loads the HIP runtime the library links against)
    lib = C.CDLL(LIB)
    lib.signmuon_debug_tile_ranges.restype = C.c_int
    # the four nanoGPT classes of a symmetric Gram launch: (M, N, K, batch, mate)
    probs = [(768, 768, 2304, 96, 0), (768, 768, 768, 96, 0), (768, 768, 3072, 96, 0), (768, 768, 3072, 96, 0)]
    total, xcd, begin = _tile_ranges(lib, probs, True, 256)
    assert total == 4 * 96 * 6 and begin == [0, 576, 1152, 1728]
    assert xcd[0] == 0 and xcd[8] == total and all(a <= b for a, b in zip(xcd, xcd[1:]))
    cost = []
    for x in range(8):
        c = 0.0
        for t in range(xcd[x], xcd[x + 1]):
            k = probs[max(i for i in range(4) if begin[i] <= t)][2]
            c += k / 64 + 6.0
        cost.append(c)
    assert max(cost) <= 1.02 * (sum(cost) / 8) + 60.0          # within a tile of the mean
    # equal problems, no symmetry, small tile: equal counts
    total, xcd, _ = _tile_ranges(lib, [(256, 512, 256, 8, 0)], False, 128)
    assert total == 2 * 4 * 8 and [b - a for a, b in zip(xcd, xcd[1:])] == [8] * 8
    # a leader with a mate owns the tiles of both; the mate's range is empty and sits at the leader's end
    total, xcd, begin = _tile_ranges(lib, [(768, 768, 768, 10, 1), (768, 768, 768, 10, 0), (512, 512, 512, 3, 0)], True, 256)
    assert begin == [0, 120, 120] and total == 120 + 3 * 3
    assert lib.signmuon_debug_tile_ranges(0, None, None, None, None, None, 1, 256, None, None) == -1


def test_gemm_tile_order_lists_every_tile_once_and_keeps_neighbours_on_few_panels():
    """Host logic of the GEMM kernels' tile decode: the list of one matrix names every tile of the grid (of its
    upper triangle for a symmetric output) exactly once, small grids keep the plain column-by-column order, and
    on a large grid a run of 32 list neighbours touches few operand panels (row panels of A plus column panels
    of B), which is what lets the tiles an XCD runs together share their panels in its L2."""
    import ctypes as C
    import torch  # noqa: F401
    lib = C.CDLL(LIB)
    f = lib.signmuon_debug_tile_of
    f.restype = C.c_int
    f.argtypes = [C.c_int] * 5 + [C.POINTER(C.c_int)] * 2

    def order(tm_n, tn_n, sym, ts):
        total = tm_n * (tm_n + 1) // 2 if sym else tm_n * tn_n
        out = []
        for t in range(total):
            a, b = C.c_int(-1), C.c_int(-1)
            assert f(t, tm_n, tn_n, int(sym), ts, C.byref(a), C.byref(b)) == 0
            out.append((a.value, b.value))
        return out

    for ts in (128, 256):
        for T in list(range(1, 20)) + [43, 64]:
            tiles = order(T, T, True, ts)
            assert sorted(tiles) == sorted((m, n) for n in range(T) for m in range(n + 1)), (ts, T)
        for tm_n, tn_n in [(1, 1), (3, 12), (12, 3), (16, 43), (43, 16), (5, 7), (9, 1), (1, 9), (17, 17), (8, 32)]:
            tiles = order(tm_n, tn_n, False, ts)
            assert sorted(tiles) == sorted((m, n) for m in range(tm_n) for n in range(tn_n)), (ts, tm_n, tn_n)
    # a grid of one band is listed column by column, rows fastest
    assert order(3, 3, True, 256) == [(0, 0), (0, 1), (1, 1), (0, 2), (1, 2), (2, 2)]
    assert order(3, 4, False, 256) == [(m, n) for n in range(4) for m in range(3)]
    # locality on a large grid of a general product: a run of 32 neighbours of the list (what an XCD works on at
    # one time) touches about 4 row panels of A and 8 or 9 column panels of B, not 16 + 2
    for tiles in (order(16, 43, False, 256), order(43, 16, False, 256)):
        counts = sorted(len({m for m, _ in tiles[i:i + 32]}) + len({n for _, n in tiles[i:i + 32]})
                        for i in range(0, len(tiles) - 31))
        assert counts[len(counts) // 2] <= 13 and counts[-1] <= 18, (counts[len(counts) // 2], counts[-1])
    # bad arguments
    a, b = C.c_int(), C.c_int()
    assert f(6, 3, 3, 1, 256, C.byref(a), C.byref(b)) == -1
    assert f(0, 3, 4, 1, 256, C.byref(a), C.byref(b)) == -1
    assert f(0, 3, 3, 0, 64, C.byref(a), C.byref(b)) == -1


def test_two_step_recurrence_coefficients_reproduce_two_newton_schulz_steps():
    """Host logic of the regrouped Newton-Schulz iteration (Alg. PolarNS with c = 0): on an eigenvalue x of
    the Gram matrix, two steps multiply Y by Q_1 Q_0 with Q_0 = a + b x and Q_1 = a + b x Q_0^2.  The
    library forms that quartic as b^4 E (E + u) + g x + a^2 with E = x (x + h); check the five
    coefficients it uses against the two explicit steps."""
    import ctypes as C
    import numpy as np
    import torch  # noqa: F401  (loads the HIP runtime the library links against)
    lib = C.CDLL(LIB)
    lib.signmuon_debug_pair_coefficients.restype = None
    lib.signmuon_debug_pair_coefficients.argtypes = [C.c_float, C.c_float, C.POINTER(C.c_float)]
    x = np.linspace(0.0, 1.6, 161)
    for a, b in [(1.5, -0.5), (1.25, -0.4), (1.4, -0.45), (1.0, -0.3), (1.5, 0.25)]:
        out = (C.c_float * 5)()
        lib.signmuon_debug_pair_coefficients(a, b, out)
        h, u, b4, g, a2 = [float(v) for v in out]
        q0 = a + b * x
        q1 = a + b * (x * q0 * q0)
        e = x * (x + h)
        got = b4 * e * (e + u) + g * x + a2
        assert np.allclose(got, q1 * q0, rtol=0, atol=2e-5 * max(1.0, np.abs(q1 * q0).max())), (a, b)
    # the paper's coefficients give exactly representable values
    lib.signmuon_debug_pair_coefficients(1.5, -0.5, out)
    assert [float(v) for v in out] == [-4.5, 6.75, 0.0625, -0.5390625, 2.25]
