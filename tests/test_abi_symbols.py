"""The C-ABI library builds, loads, and exports every symbol include/cassandra.h declares.
No compute calls (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "cassandra.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(cas_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    from paper_2605_26558_amd import binding as B
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    lib = ctypes.CDLL(B.LIB_PATH)
    names = _declared()
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), f"{n} declared in cassandra.h but not exported"
    # the binding mirrors the header one to one
    assert sorted(B.exported_names()) == names


def test_host_only_calls_work_without_a_gpu():
    from paper_2605_26558_amd import binding as B
    d = B.cas_weight_desc(4096, 4096, 600, 4)
    assert (d.K, d.bw, d.sw, d.lw, d.pw) == (2458, 128, 922, 308, 819)
    assert d.spec_bytes % 256 == 0 and d.off_spec % 256 == 0 and d.off_pruned % 256 == 0
    assert B.cas_accept([1, 2, 3], [1, 2, 9, 4]) == (2, [1, 2, 9])
    assert B.cas_accept([], [7]) == (0, [7])
    import itertools
    from oracle import cassandra_oracle as O
    for gamma in range(0, 4):
        for ratios in itertools.product([0.0, 0.3, 1.0, 2.5], repeat=gamma):
            for rs in itertools.product([0.0, 0.29, 0.31, 0.99], repeat=gamma):
                p, q = [x * 0.4 for x in ratios], [0.4] * gamma
                assert B.cas_accept_sampling(p, q, rs) == O.accept_sampling(p, q, rs)
    # layout of the shared-exponent form: 9-t bits per kept value, one exponent byte per bitmap word
    m = B.cas_mx_plan(d)
    assert (m.fw, m.ew) == ((2458 * 5 + 31) // 32, 128)
    assert m.off_sexp % 256 == 0 and m.off_field % 256 == 0 and m.off_pruned % 256 == 0
    assert m.spec_bytes >= m.off_field + 4096 * m.fw * 4 and m.verif_bytes >= m.off_pruned + 4096 * d.pw * 4
    import pytest
    with pytest.raises(B.CasError):
        B.cas_weight_desc(8, 8, 600, 9)
    with pytest.raises(B.CasError):
        B.cas_weight_desc(8, 8, 600, 4, exp_mode=1)


def test_objective_and_grid_search_against_oracle_and_closed_forms():
    """Eq. 2 and the grid search of Sec. 7.2.2 (host-only entry points): the value printed
    for the default configuration, scaling laws of the formula, and the oracle on random grids."""
    import numpy as np
    from oracle import cassandra_oracle as O
    from paper_2605_26558_amd import binding as B
    # default configuration, 4096 weights, no cache term: 4096 * 0.6 * 12 = 29491.2 bits (golden file)
    j = B.cas_objective(1.0, 4096.0, 600, 4, 0.0, 600, 4)
    assert abs(1.0 / j - 29491.2) < 1e-9
    assert abs(O.objective_j(1.0, 4096.0, 0.6, 4, 0.0, 0.6, 4) - j) < 1e-18
    # linear in alpha; halving every size doubles J; nothing truncated, nothing pruned = B bits per value
    assert abs(B.cas_objective(0.5, 4096.0, 600, 4, 100.0, 500, 2) * 2 - B.cas_objective(1.0, 4096.0, 600, 4, 100.0, 500, 2)) < 1e-18
    assert abs(B.cas_objective(0.7, 2048.0, 600, 4, 50.0, 500, 2) - 2 * B.cas_objective(0.7, 4096.0, 600, 4, 100.0, 500, 2)) < 1e-18
    assert abs(1.0 / B.cas_objective(1.0, 10.0, 1000, 0, 6.0, 1000, 0) - 16 * 16.0) < 1e-12
    rng = np.random.Generator(np.random.Philox(4))
    keeps, truncs = [700, 600, 500, 400], [0, 1, 2, 3, 4, 5]          # the grid of Sec. 7.2.2
    for _ in range(50):
        alpha = rng.uniform(0.2, 0.95, size=(4, 6))
        s_w, s_kv = float(rng.integers(1, 10**6)), float(rng.integers(0, 10**6))
        got = B.cas_tune_grid(alpha.tolist(), keeps, truncs, s_w, s_kv, 600, 4)
        ref = O.tune_grid(alpha, [k / 1000.0 for k in keeps], truncs, s_w, s_kv, 0.6, 4)
        vals = np.array([[O.objective_j(alpha[i][j], s_w, keeps[i] / 1000.0, truncs[j], s_kv, 0.6, 4)
                          for j in range(6)] for i in range(4)])
        assert got == ref == tuple(int(v) for v in np.unravel_index(np.argmax(vals), vals.shape))
    with __import__("pytest").raises(B.CasError):
        B.cas_objective(1.0, 0.0, 600, 4, 0.0, 600, 4)


def test_header_is_plain_c_and_host_calls_work_from_c(tmp_path):
    """include/cassandra.h compiles as strict C99 and a C program linked against the library
    can use the host-only entry points (no GPU touched)."""
    import shutil
    import subprocess
    from paper_2605_26558_amd import binding as B
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    gcc = shutil.which("gcc")
    assert gcc, "gcc is part of the image"
    exe = tmp_path / "abi_host_calls"
    libdir = os.path.dirname(B.LIB_PATH)
    cmd = [gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c", "abi_host_calls.c"), "-o", str(exe),
           "-L", libdir, "-l:" + os.path.basename(B.LIB_PATH), "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "abi host calls ok" in r.stdout


def test_speed_model_and_measured_format_search_against_oracle():
    """cas_speed_model / cas_tune_measured (host only) against the oracle on random grids, and
    the error paths."""
    import numpy as np
    import pytest
    from oracle import cassandra_oracle as O
    from paper_2605_26558_amd import binding as B
    rng = np.random.Generator(np.random.Philox(11))
    for _ in range(50):
        a, g = float(rng.random()), int(rng.integers(0, 9))
        td, tv, tp = (float(x) for x in rng.random(3) + 0.1)
        got, ref = B.cas_speed_model(a, g, td, tv, tp), O.speed_model(a, g, td, tv, tp)
        assert max(abs(x - y) for x, y in zip(got, ref)) < 1e-12
    assert B.cas_speed_model(1.0, 4, 1.0, 2.0, 2.0)[0] == 5.0
    for _ in range(20):
        nk, nt, g = int(rng.integers(1, 5)), int(rng.integers(1, 7)), int(rng.integers(1, 8))
        al, td, tv = rng.random((nk, nt)), rng.random((nk, nt)) + 0.1, rng.random((nk, nt)) + 0.5
        best, rates = B.cas_tune_measured(al.tolist(), td.tolist(), tv.tolist(), g)
        assert best == O.tune_measured(al, td, tv, g)
        want = [[O.speed_model(al[i][j], g, td[i][j], tv[i][j], 0.0)[1] for j in range(nt)] for i in range(nk)]
        assert np.abs(np.array(rates) - np.array(want)).max() < 1e-12
    with pytest.raises(B.CasError):
        B.cas_speed_model(1.5, 4, 1.0, 2.0, 2.0)
    with pytest.raises(B.CasError):
        B.cas_speed_model(0.5, 4, 1.0, 0.0, 2.0)


def test_kv_geometry_of_both_exponent_modes_in_closed_form():
    """cas_kv_desc_init (host only): stream widths and tile sizes of the raw and the shared-exponent
    cache against the sizes the layout description in the header gives, for several formats; a
    mode the cache has no kernels for is refused as unsupported."""
    from paper_2605_26558_amd import binding as B
    lib = B._lib()
    words = lambda bits: (bits + 31) // 32
    up256 = lambda n: (n + 255) // 256 * 256
    for keep, t in ((600, 4), (1000, 0), (250, 7), (0, 4)):
        K = min(128, max(0, (keep * 128 + 500) // 1000))
        for mode, fw_bits, extra in ((B.CAS_EXP_RAW, 16 - t, 0), (B.CAS_EXP_SHARED, 9 - t, 1)):
            d = B.cas_kv_desc()
            d.n_layers, d.n_kv_heads, d.head_dim, d.page_tokens = 3, 2, 128, 64
            d.n_pages, d.max_seqs, d.max_pages_per_seq = 5, 1, 5
            d.fmt = B.cas_fmt(keep, t, mode)
            assert lib.cas_kv_desc_init(ctypes.byref(d)) == B.CAS_OK
            assert (d.K, d.sw, d.lw, d.pw) == (K, words(K * fw_bits), words(K * t), words((128 - K) * 16))
            assert d.tile_spec_bytes == up256(64 * (4 + extra + d.sw) * 4)
            assert d.tile_verif_bytes == up256(64 * (d.lw + d.pw) * 4)
            tiles = 3 * 5 * 2 * 2
            assert d.spec_pool_bytes >= tiles * d.tile_spec_bytes and d.verif_pool_bytes >= tiles * d.tile_verif_bytes
    d.fmt = B.cas_fmt(600, 4, 1)
    assert lib.cas_kv_desc_init(ctypes.byref(d)) == B.CAS_ENOTSUP
