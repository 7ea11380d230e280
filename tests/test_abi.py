"""The C-ABI boundary without a GPU: libpsa.so loads, exports every function include/psa.h declares,
and rejects on the host what the header says it rejects (nothing is enqueued on those paths, so no
device is needed).  No compute call is made here."""
import ctypes as C
import os
import re

import pytest

import paper_2503_00392_amd as psa
from paper_2503_00392_amd import binding as pb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "psa.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(psa.library_path()):
        from paper_2503_00392_amd import build
        build.build()
    return psa.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(psa_[a-z_]+)\s*\(", text)))


def test_header_declares_the_named_entry_points():
    names = declared_functions()
    for want in ("psa_build_block_metadata", "psa_decode_attention", "psa_dense_attention", "psa_topk_attention",
                 "psa_decode_workspace_bytes", "psa_dense_workspace_bytes", "psa_read_device_error",
                 "psa_status_string"):
        assert want in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"libpsa.so does not export {name}"


def test_python_binding_mirrors_the_header():
    for name in declared_functions():
        assert hasattr(psa, name[len("psa_"):]), f"binding lacks {name}"


def test_status_strings(lib):
    assert [psa.status_string(i) for i in range(5)] == [
        "PSA_OK", "PSA_ERR_INVALID_ARG", "PSA_ERR_UNSUPPORTED", "PSA_ERR_WORKSPACE_TOO_SMALL",
        "PSA_ERR_LAUNCH"]
    assert psa.status_string(99) == "PSA_ERR_UNKNOWN"


def _desc(**kw):
    base = dict(batch=2, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16, num_pages=64,
                max_blocks_per_seq=32, dtype=0, k_pool=0x1000, v_pool=0x2000, block_table=0x3000,
                ctx_lens=0x4000)
    base.update(kw)
    return pb._KvDesc(**base)


def _decode(lib, d, threshold=0.9, m=1, q=0x10, meta=0x20, out=0x30, nsel=0x40, mass=0x50, ws=0x60,
            ws_bytes=1 << 40, tuning=None, scorer=0):
    return lib.psa_decode_attention(C.byref(d), q, meta, threshold, m, scorer, out, nsel, mass, None, None,
                                    None, None, None, C.byref(tuning) if tuning else None, ws, ws_bytes, None)


def test_workspace_sizes(lib):
    d = _desc()
    n = lib.psa_decode_workspace_bytes(C.byref(d), None)
    assert n > 0 and n % 256 == 0
    bigger = lib.psa_decode_workspace_bytes(C.byref(_desc(max_blocks_per_seq=64)), None)
    assert bigger > n
    assert lib.psa_dense_workspace_bytes(C.byref(d)) > 0
    assert lib.psa_decode_workspace_bytes(None, None) == 0
    assert lib.psa_decode_workspace_bytes(C.byref(_desc(head_dim=64)), None) == 0
    assert lib.psa_decode_workspace_bytes(C.byref(_desc(max_blocks_per_seq=8193)), None) == 0
    assert lib.psa_dense_workspace_bytes(C.byref(_desc(num_q_heads=30))) == 0


@pytest.mark.parametrize("kw,want", [
    (dict(head_dim=64), 2), (dict(page_size=32), 2), (dict(dtype=2), 2),
    (dict(num_q_heads=24), 2),            # group of 3 is not built
    (dict(num_q_heads=30), 1),            # not a multiple of the KV heads
    (dict(batch=-1), 1), (dict(num_kv_heads=0), 1), (dict(k_pool=None), 1), (dict(v_pool=None), 1),
    (dict(block_table=None), 1), (dict(ctx_lens=None), 1),
    (dict(max_blocks_per_seq=8193), 2), (dict(max_blocks_per_seq=0), 1),
])
def test_decode_rejects_bad_descriptors_on_the_host(lib, kw, want):
    assert _decode(lib, _desc(**kw)) == want


def test_decode_rejects_bad_scalars_and_null_buffers(lib):
    d = _desc()
    assert _decode(lib, d, threshold=float("nan")) == 1
    assert _decode(lib, d, threshold=-0.01) == 1
    assert _decode(lib, d, threshold=1.01) == 1
    assert _decode(lib, d, m=0) == 1
    assert _decode(lib, d, scorer=3) == 1 and _decode(lib, d, scorer=-1) == 1
    for name in ("q", "meta", "out", "nsel", "mass", "ws"):
        assert _decode(lib, d, **{name: None}) == 1, name
    assert _decode(lib, d, ws_bytes=1024) == 3
    T = pb._Tuning        # chunk_blocks, window_chunks, spin_limit, force_bitonic, depth_hint, events
    assert _decode(lib, d, tuning=T(7, 0, 0, 0, None, None)) == 1       # too small
    assert _decode(lib, d, tuning=T(10, 0, 0, 0, None, None)) == 1      # not a multiple of 4
    assert _decode(lib, d, tuning=T(68, 0, 0, 0, None, None)) == 1      # too large
    assert _decode(lib, d, tuning=T(0, -1, 0, 0, None, None)) == 1
    assert _decode(lib, d, tuning=T(0, 0, 0, 2, None, None)) == 1
    assert _decode(lib, d, tuning=T(0, 0, -1, 0, None, None)) == 1
    assert lib.psa_decode_attention(None, 1, 1, 0.5, 1, 0, 1, 1, 1, None, None, None, None, None, None, 1,
                                    1 << 30, None) == 1
    assert lib.psa_topk_attention(C.byref(d), 0x10, 0x20, 0, 0, 0x30, 0x40, 0x50, None, None, None, None, None,
                                  None, 0x60, 1 << 40, None) == 1          # budget below one block
    assert lib.psa_topk_attention(C.byref(d), 0x10, 0x20, 4, 0, 0x30, 0x40, 0x50, None, None, None, None, None,
                                  None, 0x60, 64, None) == 3


def test_empty_batch_is_ok_and_enqueues_nothing(lib):
    d = _desc(batch=0, block_table=None, ctx_lens=None)
    assert _decode(lib, d, q=None, out=None, nsel=None, mass=None, ws=None, ws_bytes=0) == 0
    assert lib.psa_dense_attention(C.byref(d), None, None, None, None, 0, None) == 0


def test_dense_and_metadata_reject_on_the_host(lib):
    d = _desc()
    assert lib.psa_dense_attention(C.byref(d), None, 0x10, None, 0x20, 1 << 40, None) == 1
    assert lib.psa_dense_attention(C.byref(d), 0x10, 0x20, None, 0x30, 16, None) == 3
    assert lib.psa_dense_attention(C.byref(_desc(head_dim=256)), 0x10, 0x20, None, 0x30, 1 << 40, None) == 2
    assert lib.psa_build_block_metadata(C.byref(d), None, None, None, 0, None) == 1
    assert lib.psa_build_block_metadata(C.byref(d), 0x10, None, None, 3, None) == 1     # count without a list
    assert lib.psa_build_block_metadata(C.byref(d), 0x10, None, None, -1, None) == 1
    assert lib.psa_build_block_metadata(C.byref(d), 0x10, None, 0x20, 0, None) == 0     # empty list: nothing to do
    assert lib.psa_build_block_metadata(C.byref(_desc(dtype=5)), 0x10, None, None, 0, None) == 2
    assert lib.psa_build_block_means(C.byref(d), None, None, None, 0, None) == 1
    assert lib.psa_build_block_means(C.byref(d), 0x10, None, None, 3, None) == 1        # count without a list
    assert lib.psa_build_block_means(C.byref(d), 0x10, None, 0x20, 0, None) == 0        # empty list: nothing to do
    assert lib.psa_build_block_means(C.byref(_desc(dtype=5)), 0x10, None, None, 0, None) == 2
    assert lib.psa_read_device_error(None, None, None) == 1


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(pb, "_lib", None)
    monkeypatch.setattr(pb, "_LIB_PATH", str(tmp_path / "libpsa.so"))
    with pytest.raises(FileNotFoundError):
        pb.load_library()


def test_tier_state_sizes(lib):
    # header + slice table + two slot tables + the slices' staging entries, each rounded up to 256 bytes; 0 for
    # sizes out of range
    assert psa.tier_state_bytes(1, 1) == 256 + 4 * 256
    assert psa.tier_state_bytes(1000, 100) == 256 + 4096 + 2 * 512 + 4096
    # a staging buffer: header, one id per entry (rounded up to 256 bytes), 8 KiB per entry
    assert psa.tier_staging_bytes(1) == 256 + 256 + 8192
    assert psa.tier_staging_bytes(1000) == 256 + 4096 + 1000 * 8192
    assert psa.tier_staging_bytes(0) == 0 and psa.tier_staging_bytes((1 << 24) + 1) == 0
    for bad in ((0, 1), (1, 0), (-5, 3), (1 << 31, 1), (1, 1 << 31)):
        assert psa.tier_state_bytes(*bad) == 0
    # a descriptor without a tier has no update scratch
    assert lib.psa_tier_update_workspace_bytes(C.byref(_desc())) == 0


def test_binding_structs_have_the_layout_of_the_header(tmp_path):
    """The ctypes mirrors of psa_kv_desc, psa_tuning and psa_tier against what a C compiler makes of
    include/psa.h: total sizes and the offset of every field."""
    import subprocess
    from paper_2503_00392_amd import binding as b
    structs = {"psa_kv_desc": b._KvDesc, "psa_tuning": b._Tuning, "psa_tier": b._Tier}
    lines = ['#include <stdio.h>', '#include <stddef.h>', f'#include "{HEADER}"', 'int main(void) {']
    for cname, ct in structs.items():
        lines.append(f'  printf("{cname} %zu\\n", sizeof({cname}));')
        for fname, _ in ct._fields_:
            lines.append(f'  printf("{cname}.{fname} %zu\\n", offsetof({cname}, {fname}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-o", str(exe), str(src)], check=True)
    got = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for cname, ct in structs.items():
        assert int(got[cname]) == C.sizeof(ct), cname
        for fname, _ in ct._fields_:
            assert int(got[f"{cname}.{fname}"]) == getattr(ct, fname).offset, f"{cname}.{fname}"


def test_static_entry_point_rejects_on_the_host_before_it_touches_a_gpu(lib):
    """psa_decode_attention_static: what does not fit its array, a bad descriptor or a second tier come back as
    codes with no device involved (this test runs without one)."""
    def call(d, threshold=0.9, m=1):
        return lib.psa_decode_attention_static(C.byref(d), 0x10, 0x20, threshold, m, 0, 0x30, 0x40, 0x50, None, None,
                                               None, None, None, None)
    big = _desc(batch=8, num_pages=8 * 8192, max_blocks_per_seq=8192)
    assert lib.psa_decode_workspace_bytes(C.byref(big), None) > pb.STATIC_SCRATCH_BYTES
    assert call(big) == 3
    assert call(_desc(head_dim=64)) == 2
    assert call(_desc(num_q_heads=30)) == 1
    assert call(_desc(batch=0)) == 0
    header = open(HEADER).read()
    assert f"#define PSA_STATIC_SCRATCH_BYTES ({pb.STATIC_SCRATCH_BYTES >> 20}u << 20)" in header
