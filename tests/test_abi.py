"""The C-ABI library loads on a machine without a GPU and exports every symbol include/lsq.h
declares; host-side error paths return codes without touching a device."""
import ctypes
import os
import re

import pytest

import lsq_synth as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2010_13887_amd as lsq
    if not os.path.exists(lsq.library_path()):
        from paper_2010_13887_amd import build
        build.build(verbose=False)
    return lsq.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "lsq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(lsq_[a-z0-9_]+)\s*\(", header))
    assert {"lsq_init", "lsq_encode", "lsq_decode_step", "lsq_get_beams", "lsq_workspace_bytes"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} is declared in lsq.h but not exported"


def test_host_side_errors(lib):
    import paper_2010_13887_amd as lsq
    w = S.workload("tiny")
    blob = w.blob()
    assert lsq.lsq_workspace_bytes(blob, 2, 4, 8) > len(blob)
    # the plan grows with every maximum
    assert lsq.lsq_workspace_bytes(blob, 4, 4, 8) > lsq.lsq_workspace_bytes(blob, 2, 4, 8)
    assert lsq.lsq_workspace_bytes(blob, 2, 4, 16) > lsq.lsq_workspace_bytes(blob, 2, 4, 8)
    for bad in (blob[:100], b"X" + blob[1:], blob[:8] + b"\x07" + blob[9:]):
        with pytest.raises(lsq.LsqError):
            lsq.lsq_workspace_bytes(bad, 2, 4, 8)
    for args in ((0, 4, 8), (2, 0, 8), (2, 9, 8), (2, 4, 0)):
        with pytest.raises(lsq.LsqError):
            lsq.lsq_workspace_bytes(blob, *args)
    n = ctypes.c_size_t()
    assert lib.lsq_workspace_bytes(None, 0, 2, 4, 8, ctypes.byref(n)) == -1          # LSQ_E_ARG
    assert lib.lsq_workspace_bytes(blob, len(blob), 2, 4, 8, None) == -1
    lsq.lsq_free()
    assert lib.lsq_decode_step() == -2 and b"lsq_encode" in lib.lsq_last_error()       # LSQ_E_STATE
    assert lib.lsq_init(blob, len(blob), 2, 4, 8) == -2                                # no workspace yet
    assert lib.lsq_set_workspace(None, 0, None) == -1
    assert lib.lsq_set_workspace(ctypes.c_void_p(3), 1024, None) == -1                 # misaligned
    # unsupported model variants are refused from the header alone
    import struct
    hdr = bytearray(blob[:256])
    struct.pack_into("<i", hdr, 12, 1)                                                 # arch = decoder-only
    assert lib.lsq_workspace_bytes(bytes(hdr), 256, 2, 4, 8, ctypes.byref(n)) == -3    # LSQ_E_BLOB


def test_blob_writer_and_oracle_reader_agree():
    from oracle import lsq_oracle as O
    hp = S.HParams(n_enc=2, n_dec=1, d_model=16, n_heads=2, d_ffn=24, vocab=11, max_pos=8, dtype=1)
    blob = S.make_blob(hp, overrides={"dec0.Wkv_c": __import__("numpy").arange(16 * 32).reshape(16, 32) / 64.0})
    m = O.Model(blob)
    assert (m.d, m.F, m.V, m.n_enc, m.n_dec, m.H) == (16, 24, 11, 2, 1, 2)
    assert m.dec[0]["Wkv_c"][3, 5] == (3 * 32 + 5) / 64.0
    assert len(S.tensor_list(hp)) == 1 + 12 * 2 + 20
    assert m.enc[1]["ln2_g"].tolist() == [1.0] * 16 and m.enc[1]["ln2_b"].tolist() == [0.0] * 16


def test_corrupt_headers_are_refused_not_trusted(lib):
    """Random damage to the 256-byte header: lsq_workspace_bytes (host only) either refuses the blob or
    reports a plan no smaller than the blob itself; it never crashes or overflows into nonsense."""
    import numpy as np
    rng = np.random.default_rng(7)
    n = ctypes.c_size_t()
    for base in (S.workload("tiny").blob(),
                 S.make_blob(S.HParams(arch=1, n_enc=0, n_dec=1, d_model=16, n_heads=1, d_ffn=16, vocab=20, max_pos=8, act=1,
                                       norm=1, sample_topk=4, sample_topp=0.5))):
        assert lib.lsq_workspace_bytes(base, len(base), 2, 1, 8, ctypes.byref(n)) == 0 and n.value > len(base)
        ok = refused = 0
        for trial in range(400):
            hdr = bytearray(base[:256])
            for _ in range(int(rng.integers(1, 4))):
                off = int(rng.integers(8, 104))
                kind = int(rng.integers(0, 3))
                if kind == 0:
                    hdr[off] = int(rng.integers(0, 256))
                elif kind == 1:
                    hdr[off - off % 4: off - off % 4 + 4] = int(rng.integers(-2**31, 2**31)).to_bytes(4, "little", signed=True)
                else:
                    hdr[off - off % 4: off - off % 4 + 4] = int(rng.choice([0, -1, 1, 2**31 - 1, 65536, 65537])).to_bytes(
                        4, "little", signed=True)
            blob = bytes(hdr) + base[256:]
            rc = lib.lsq_workspace_bytes(blob, len(blob), 2, 1, 8, ctypes.byref(n))
            assert rc in (0, -1, -3), rc
            if rc == 0:
                ok += 1
                assert len(base) <= n.value < (1 << 40)       # accepted only if the shapes still add up to the stated size
            else:
                refused += 1
                assert len(lib.lsq_last_error()) > 0
        assert refused > 100                                  # most damage is caught by a range or size check
