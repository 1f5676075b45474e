"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and the host
logic (configuration checks, memory sizing) behaves.  No compute call is made here."""
import ctypes as C
import os
import re

import pytest

from paper_2201_05500_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(**kw):
    d = dict(capacity_rows=1 << 16, dim=8, load_factor=0.5, n_replicas=1, lr=1e-3, beta1=0.9,
             beta2=0.999, eps=1e-8, init_seed=0, init_std=0.01, flags=0)
    d.update(kw)
    return B.ctr_config(*[d[f[0]] for f in B.ctr_config._fields_])


def test_library_exports_every_declared_symbol():
    from paper_2201_05500_amd import binding_mlp as BM
    lib = C.CDLL(B.LIB_PATH)
    for hdr, exported in (("ctr_sparse.h", B.EXPORTED), ("ctr_mlp.h", BM.EXPORTED)):
        header = open(os.path.join(ROOT, "include", hdr)).read()
        declared = set(re.findall(r"^\s*(?:int|size_t)\s+(ctr_\w+)\s*\(", header, re.M))
        assert declared == set(exported), hdr
        for name in declared:
            assert hasattr(lib, name), name


def test_mlp_host_logic():
    from paper_2201_05500_amd import binding_mlp as BM
    L = BM.lib()
    cfg = BM.make_config(19200, [1024, 512, 256])
    n = 19200 * 1024 + 1024 + 1024 * 512 + 512 + 512 * 256 + 256 + 256 + 1
    assert L.ctr_mlp_n_params(C.byref(cfg)) == n == 20318209
    assert L.ctr_mlp_bytes(C.byref(cfg)) >= n * (4 * 3 + 2)
    assert L.ctr_mlp_workspace_bytes(C.byref(cfg), 16384) >= 16384 * 19200 * 2
    assert L.ctr_mlp_workspace_bytes(C.byref(cfg), 100) == 0          # batch must be a multiple of 8
    assert L.ctr_mlp_workspace_bytes(C.byref(cfg), (1 << 20) + 8) == 0  # and at most CTR_MLP_MAX_BATCH
    for bad in (BM.make_config(100, [8]), BM.make_config(64, []), BM.make_config(64, [12]),
                BM.make_config(64, [8], n_replicas=2), BM.make_config(64, [8], lr=0.0)):
        assert L.ctr_mlp_bytes(C.byref(bad)) == 0
    out = C.c_void_p()
    assert L.ctr_mlp_create(C.byref(BM.make_config(64, [12])), 256, 1 << 30, None, C.byref(out)) == B.CTR_E_INVAL
    assert L.ctr_mlp_destroy(None) == B.CTR_E_INVAL


def test_config_struct_matches_header_layout():
    # uint64, uint32, float, uint32, 4 floats, uint64, float, uint32 with natural alignment
    assert C.sizeof(B.ctr_config) == 56
    assert B.ctr_config.init_seed.offset == 40 and B.ctr_config.flags.offset == 52


def test_table_bytes_accounts_for_every_array():
    R, D = 1 << 16, 8
    n = B.ctr_table_bytes(_cfg())
    slots = (1 << 17) * 16
    assert n >= slots + R * 8 + R * 4 + R * 3 * D * 4
    assert n < slots + R * 8 + R * 4 + R * 3 * D * 4 + 4096
    k = B.ctr_table_bytes(_cfg(n_replicas=8, flags=B.CTR_F_KSTEP))
    assert k - n >= 7 * R * 3 * D * 4 + R * D * 4
    # load factor decides the number of index slots (next power of two of R / lf)
    assert B.ctr_table_bytes(_cfg(load_factor=0.25)) - n == (1 << 17) * 16
    assert B.ctr_table_bytes(_cfg(load_factor=0.0)) == n            # 0 selects 0.5
    # AdaGrad rows hold two arrays instead of three; the prose merge needs no shared-denominator array
    assert n - B.ctr_table_bytes(_cfg(flags=B.CTR_F_ADAGRAD)) == R * D * 4
    assert k - B.ctr_table_bytes(_cfg(n_replicas=8, flags=B.CTR_F_KSTEP | B.CTR_F_KSTEP_PROSE)) == R * D * 4


@pytest.mark.parametrize("bad", [
    dict(dim=0), dict(dim=6), dict(dim=260), dict(capacity_rows=0), dict(capacity_rows=(1 << 30) + 1),
    dict(n_replicas=0), dict(n_replicas=32), dict(load_factor=0.95), dict(load_factor=-1.0),
    dict(flags=16), dict(flags=B.CTR_F_KSTEP_PROSE), dict(flags=B.CTR_F_ADAGRAD | B.CTR_F_KSTEP),
    dict(flags=B.CTR_F_ADAGRAD, n_replicas=2), dict(flags=B.CTR_F_BIAS_CORRECTION | B.CTR_F_KSTEP),
    dict(n_replicas=2), dict(lr=0.0), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=0.0),
])
def test_invalid_configurations_are_rejected(bad):
    assert B.ctr_table_bytes(_cfg(**bad)) == 0
    assert B.ctr_workspace_bytes(_cfg(**bad), 1000, 10) == 0
    out = C.c_void_p()
    st = B.lib().ctr_table_create(C.byref(_cfg(**bad)), 256, 1 << 30, None, C.byref(out))
    assert st == B.CTR_E_INVAL


def test_workspace_bytes_grow_with_keys_and_dim():
    a = B.ctr_workspace_bytes(_cfg(), 10000, 100)
    b = B.ctr_workspace_bytes(_cfg(), 20000, 100)
    c = B.ctr_workspace_bytes(_cfg(dim=64), 10000, 100)
    assert 0 < a < b and a < c
    assert B.ctr_workspace_bytes(_cfg(), 0, 0) >= 256
    assert B.ctr_workspace_bytes(_cfg(), 1 << 31, 10) == 0           # n_keys limit


def test_workspace_bytes_never_shrink_with_the_batch_size():
    """The work geometry changes at 2, 4 and 8 Mi occurrences (shorter spans below each threshold need more
    partial sums): a workspace sized for max_keys must cover every smaller batch."""
    for dim in (16, 64):
        sizes = [1, 1000, (1 << 20), (2 << 20) - 1, 2 << 20, (3 << 20), (4 << 20) - 1, 4 << 20, (6 << 20),
                 (8 << 20) - 1, 8 << 20, 12 << 20, 40 << 20]
        need = [B.ctr_workspace_bytes(_cfg(dim=dim), n, 10) for n in sizes]
        assert all(a <= b for a, b in zip(need, need[1:])), (dim, need)
        assert all(n > 0 for n in need)


def test_null_and_misaligned_arguments():
    L = B.lib()
    out = C.c_void_p()
    assert L.ctr_table_create(None, 256, 1 << 30, None, C.byref(out)) == B.CTR_E_INVAL
    assert L.ctr_table_create(C.byref(_cfg()), None, 1 << 30, None, C.byref(out)) == B.CTR_E_INVAL
    assert L.ctr_table_create(C.byref(_cfg()), 264, 1 << 30, None, C.byref(out)) == B.CTR_E_INVAL
    assert L.ctr_table_create(C.byref(_cfg()), 256, 1024, None, C.byref(out)) == B.CTR_E_NOMEM
    assert L.ctr_table_destroy(None) == B.CTR_E_INVAL
    assert L.ctr_kstep_merge(None, None) == B.CTR_E_INVAL
    assert L.ctr_push_adam(None, 0, None, None, 0, None) == B.CTR_E_INVAL
    assert L.ctr_last_status(None, None) == B.CTR_E_INVAL
    assert L.ctr_debug_set_geometry(None, 0, 0) == B.CTR_E_INVAL
    assert L.ctr_debug_set_push_order(None, 32, 0, 0) == B.CTR_E_INVAL


def test_headers_are_plain_c99(tmp_path):
    """The boundary is a C ABI: both headers compile as strict C99 on their own."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "hdr.c"
    src.write_text('#include "ctr_sparse.h"\n#include "ctr_mlp.h"\nint main(void) { return 0; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I" + os.path.join(root, "include"),
                           "-fsyntax-only", str(src)])


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """No CPU fallback exists: without the built HIP library the binding raises instead of computing."""
    from paper_2201_05500_amd import binding as B
    from paper_2201_05500_amd import binding_mlp as BM
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libctr_sparse.so"))
    monkeypatch.setattr(B, "_lib", None)
    with pytest.raises(RuntimeError, match="missing"):
        B.lib()
    with pytest.raises(RuntimeError, match="missing"):          # the tower's binding loads the same library
        BM.lib()
