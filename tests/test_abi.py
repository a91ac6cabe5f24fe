"""CPU-only checks of the C boundary: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "tagore_knn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tg_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2508_08744_amd import knn
    lib = knn.lib()
    names = _declared()
    assert len(names) >= 18
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(knn.EXPORTS) == names


def test_default_params_follow_the_paper():
    from paper_2508_08744_amd import knn
    p = knn.default_params(32, 12)
    assert (p.it1, p.it2) == (6, 6)            # it1 = it2 (section 7.3)
    assert p.m == 2                            # top-m unvisited neighbours, m = 2 (section 4.1)
    assert p.delta == 0.0 and p.k == 32
    p = knn.default_params(16, 7)
    assert (p.it1, p.it2, p.S) == (4, 3, 16)
    # a budget below eight rounds goes to the first phase first
    assert [(q.it1, q.it2) for q in (knn.default_params(32, i) for i in (1, 3, 4, 5, 8, 9))] == [(1, 0), (3, 0), (4, 0), (4, 1), (4, 4), (5, 4)]
    p = knn.default_params(32, 0)
    assert p.it1 + p.it2 == 16 and p.delta > 0


def test_invalid_arguments_are_rejected_on_the_host():
    from paper_2508_08744_amd import knn
    lib = knn.lib()
    bad = [
        dict(n=10, d=4, k=20),          # k >= n
        dict(n=100, d=4, k=0),
        dict(n=100, d=4, k=65),
        dict(n=100, d=0, k=5),
        dict(n=100, d=5000, k=5),
        dict(n=2**30, d=4, k=5),
        dict(n=100, d=4, k=5, metric=7),
    ]
    fake = ctypes.c_void_p(256)
    for b in bad:
        rc = lib.tg_knn_build(fake, b["n"], b["d"], b["k"], b.get("metric", 0), 4, 1, fake, None, None)
        assert rc == -1, b
        assert lib.tg_last_error()
    assert lib.tg_knn_build(None, 100, 4, 5, 0, 4, 1, fake, None, None) == -1
    assert lib.tg_knn_build(fake, 100, 4, 5, 0, 4, 1, None, None, None) == -1
    for field, val in [("C", 48), ("C", 8), ("S", 0), ("S", 33), ("R", 33), ("parts", 3), ("parts", 16), ("parts", 0), ("m", 0),
                       ("it1", 70), ("delta", 2.0), ("screen", 2), ("join_f16", 3), ("join_f16", -1)]:
        p = knn.default_params(8, 4)
        setattr(p, field, val)
        assert lib.tg_knn_workspace_bytes(1000, 16, ctypes.byref(p)) == 0, field
        h = ctypes.c_void_p()
        assert lib.tg_knn_create(ctypes.byref(h), fake, 1000, 16, ctypes.byref(p), fake, 1 << 30, None) == -1
    p = knn.default_params(8, 4)
    need = lib.tg_knn_workspace_bytes(1000, 16, ctypes.byref(p))
    assert need > 1000 * 8 * 4
    h = ctypes.c_void_p()
    assert lib.tg_knn_create(ctypes.byref(h), fake, 1000, 16, ctypes.byref(p), fake, need // 2, None) == -1
    assert b"workspace too small" in lib.tg_last_error()
    assert lib.tg_knn_create(ctypes.byref(h), fake, 1000, 16, ctypes.byref(p), ctypes.c_void_p(8), need, None) == -1
    assert lib.tg_exact_knn(fake, 100, 4, 200, 0, None, 10, fake, None, None) == -1
    assert lib.tg_knn_init(None) == -1 and lib.tg_knn_destroy(None) == 0
    # pruning entry points: (n, d, k, hops, cand_size, alpha, d_out) -> status, before anything is launched
    for a, want in [((100, 8, 16, 1, 64, 1.0, 0), -1), ((100, 8, 16, 1, 64, 1.0, 65), -1), ((100, 8, 16, 3, 64, 1.0, 8), -1),
                    ((100, 8, 16, 1, 0, 1.0, 8), -1), ((100, 8, 16, 1, 65, 1.0, 8), -1), ((100, 8, 16, 1, 64, 0.99, 8), -1),
                    ((100, 8, 16, 1, 64, float("nan"), 8), -1), ((0, 8, 16, 1, 64, 1.0, 8), -1), ((100, 0, 16, 1, 64, 1.0, 8), -1),
                    ((100, 8, 65, 1, 64, 1.0, 8), -1), ((100, 8, 65, 2, 64, 1.0, 8), -1)]:
        n, d, k, hops, cs, alpha, d_out = a
        assert lib.tg_prune_dist(fake, n, d, fake, k, hops, cs, alpha, d_out, fake, None, None) == want, a
    assert lib.tg_prune_dist(None, 100, 8, fake, 16, 1, 64, 1.0, 8, fake, None, None) == -1
    for a, want in [((100, 8, 16, 1, 64, 60.0, 0), -1), ((100, 8, 16, 3, 64, 60.0, 8), -1), ((100, 8, 16, 1, 65, 60.0, 8), -1),
                    ((100, 8, 16, 1, 64, 0.0, 8), -1), ((100, 8, 16, 1, 64, 90.01, 8), -1), ((100, 8, 16, 1, 64, -60.0, 8), -1),
                    ((100, 8, 16, 1, 64, float("nan"), 8), -1), ((100, 8, 65, 2, 64, 60.0, 8), -1)]:
        n, d, k, hops, cs, gamma, d_out = a
        assert lib.tg_prune_angle(fake, n, d, fake, k, hops, cs, gamma, d_out, fake, None, None) == want, a
    assert lib.tg_prune_angle(fake, 100, 8, None, 16, 1, 64, 60.0, 8, fake, None, None) == -1
    for a, want in [((100, 8, 16, 1, 64, 0), -1), ((100, 8, 16, 1, 64, 65), -1), ((100, 8, 16, 0, 64, 8), -1),
                    ((100, 8, 16, 1, 0, 8), -1), ((100, 8, 65, 1, 64, 8), -1), ((100, 4097, 16, 1, 64, 8), -1),
                    ((100, 8, 65, 2, 64, 8), -1)]:
        n, d, k, hops, cs, d_out = a
        assert lib.tg_prune_dispersion(fake, n, d, fake, k, hops, cs, d_out, fake, None, None) == want, a
    assert lib.tg_prune_dispersion(fake, 100, 8, fake, 16, 1, 64, 8, None, None, None) == -1
    assert lib.tg_angle_at(fake, fake, fake, fake, -1, None) == -1
    assert lib.tg_angle_at(fake, None, fake, fake, 5, None) == -1
    assert lib.tg_angle_at(None, None, None, None, 0, None) == 0
    assert lib.tg_prune_rank(fake, 100, 16, 17, fake, None, None) == -1


def test_workspace_fits_the_largest_configuration():
    # the 1e8 x 96 configuration must fit one MI355X (288 GB) together with its vectors and outputs
    from paper_2508_08744_amd import inputs, knn
    cfg = inputs.CONFIGS["C5"]
    p = knn.default_params(cfg["k"], 12, parts=8, C=64)      # (the adjacency words of one part are n / parts * 2 KB, the slots n * C * 8 B)
    ws = knn.workspace_bytes(cfg["n"], cfg["d"], p)
    total = ws + cfg["n"] * cfg["d"] * 4 + cfg["n"] * cfg["k"] * 8
    assert total < 288e9, total / 1e9


def test_missing_library_is_an_error(monkeypatch):
    from paper_2508_08744_amd import knn
    monkeypatch.setattr(knn, "_lib", None)
    monkeypatch.setattr(knn, "_LIB_PATH", "/nonexistent/libtagore_knn.so")
    with pytest.raises(RuntimeError):
        knn.lib()


def test_binding_refuses_host_tensors():
    # there is no CPU path behind the binding: tensors that are not on the device are turned away before
    # the library is called, whatever the entry point
    import torch
    from paper_2508_08744_amd import knn
    X = torch.zeros((100, 8))
    ids = torch.zeros((100, 4), dtype=torch.int32)
    for call in (lambda: knn.knn_build(X, 4), lambda: knn.knn_build_ex(X, knn.default_params(4, 2)),
                 lambda: knn.exact_knn(X, 4), lambda: knn.prune_dist(X, ids, 2), lambda: knn.prune_angle(X, ids, 2),
                 lambda: knn.prune_dispersion(X, ids, 2), lambda: knn.angle_at(X[0], X[0], X[0])):
        with pytest.raises((TypeError, ValueError)):
            call()
    with pytest.raises((TypeError, ValueError)):
        knn.prune_rank(ids, 2)
    with pytest.raises((TypeError, ValueError)):
        knn.merge_local(ids, X[:, :4].contiguous(), ids, X[:, :4].contiguous(), torch.arange(100, dtype=torch.int32))


def test_binding_structures_match_the_header(tmp_path):
    """The ctypes mirrors of tg_knn_params and tg_knn_stats have the header's sizes and field offsets
    (a C program compiled against include/tagore_knn.h prints them)."""
    import subprocess
    from paper_2508_08744_amd import knn
    src = tmp_path / "layout.c"
    fields_p = [f for f, _ in knn.Params._fields_]
    fields_s = [f for f, _ in knn.Stats._fields_]
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "tagore_knn.h"', 'int main(void) {',
             'printf("%zu %zu\\n", sizeof(tg_knn_params), sizeof(tg_knn_stats));']
    lines += ['printf("%%zu\\n", offsetof(tg_knn_params, %s));' % f for f in fields_p]
    lines += ['printf("%%zu\\n", offsetof(tg_knn_stats, %s));' % f for f in fields_s]
    lines += ['return 0; }']
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(out[0]), int(out[1])] == [ctypes.sizeof(knn.Params), ctypes.sizeof(knn.Stats)]
    want = [getattr(knn.Params, f).offset for f in fields_p] + [getattr(knn.Stats, f).offset for f in fields_s]
    assert [int(x) for x in out[2:]] == want
