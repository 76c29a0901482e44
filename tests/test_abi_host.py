"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the public header declares, and rejects bad index descriptions
before touching a device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2312_01712_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ivfpq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ivfpq_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    names = declared_symbols()
    assert len(names) >= 11
    for n in names:
        assert getattr(lib, n) is not None, n
    assert sorted(binding.SYMBOLS) == names


def _desc(**over):
    nlist, D, M, N = 4, 8, 4, 10
    arrays = dict(
        centroids=np.zeros((nlist, D), np.float32), codebooks=np.zeros((M, 256, D // M), np.float32),
        list_offsets=np.array([0, 3, 3, 7, 10], np.int64), codes=np.zeros((N, M), np.uint8))
    fields = dict(N=N, D=D, nlist=nlist, M=M, ksub=256)
    for k, v in over.items():
        if k in arrays:
            arrays[k] = v
        else:
            fields[k] = v
    d = binding._Desc(**fields, **{k: (v.ctypes.data if v is not None else None) for k, v in arrays.items()}, ids=None)
    return d, arrays


@pytest.mark.parametrize("over,status", [
    (dict(ksub=16), binding.ERR_UNSUPPORTED),
    (dict(D=9), binding.ERR_INVALID_ARGUMENT),
    (dict(M=0), binding.ERR_INVALID_ARGUMENT),
    (dict(nlist=0), binding.ERR_INVALID_ARGUMENT),
    (dict(N=-1), binding.ERR_INVALID_ARGUMENT),
    (dict(N=1 << 33), binding.ERR_UNSUPPORTED),
    (dict(metric=2), binding.ERR_INVALID_ARGUMENT),
    (dict(metric=-1), binding.ERR_INVALID_ARGUMENT),
    (dict(centroids=None), binding.ERR_INVALID_ARGUMENT),
    (dict(codes=None), binding.ERR_INVALID_ARGUMENT),
    (dict(list_offsets=np.array([0, 3, 2, 7, 10], np.int64)), binding.ERR_INVALID_ARGUMENT),
    (dict(list_offsets=np.array([1, 3, 3, 7, 10], np.int64)), binding.ERR_INVALID_ARGUMENT),
    (dict(list_offsets=np.array([0, 3, 3, 7, 9], np.int64)), binding.ERR_INVALID_ARGUMENT),
])
def test_index_create_rejects_bad_descriptions(over, status):
    lib = binding.load_library()
    d, keep = _desc(**over)
    h = ctypes.c_void_p()
    rc = lib.ivfpq_index_create(ctypes.byref(d), ctypes.byref(h))
    assert rc == status, (over, rc, binding.last_error())
    assert h.value is None and binding.last_error() != ""


def test_null_handles_are_rejected():
    lib = binding.load_library()
    assert lib.ivfpq_search_workspace_bytes(None, 10, 1, 1) == 0
    assert lib.ivfpq_search(None, None, 1, 1, 1, None, None, None, None, 0, None) == binding.ERR_INVALID_ARGUMENT
    assert lib.ivfpq_index_get_info(None, None) == binding.ERR_INVALID_ARGUMENT
    assert lib.ivfpq_set_option(b"no_such_option", 1) == binding.ERR_INVALID_ARGUMENT
    lib.ivfpq_index_destroy(None)
    assert lib.ivfpq_radius_model_create(None, None, None) == binding.ERR_INVALID_ARGUMENT
    assert lib.ivfpq_query_radii(None, None, None, 1, None, 1, ctypes.c_float(1.0), None, None) == binding.ERR_INVALID_ARGUMENT
    lib.ivfpq_radius_model_destroy(None)


def test_header_is_plain_c():
    """include/ivfpq.h must compile as C (no C++ constructs, no torch or HIP types)."""
    import subprocess
    import tempfile
    with tempfile.TemporaryDirectory() as d:
        src = os.path.join(d, "use.c")
        with open(src, "w") as f:
            f.write('#include "ivfpq.h"\n'
                    "int probe(const ivfpq_index *ix, const float *q, void *ws, size_t n) {\n"
                    "  ivfpq_scoring sc = {IVFPQ_SCORE_DISTANCE, 0, IVFPQ_SCAN_AUTO};\n"
                    "  ivfpq_radius_model_desc md = {0};\n"
                    "  (void)md;\n"
                    "  return ivfpq_search_ex(ix, q, 1, 1, 1, 0, &sc, 0, 0, ws, n, 0);\n"
                    "}\n")
        r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I",
                            os.path.join(ROOT, "include"), "-c", src, "-o", os.path.join(d, "use.o")],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: `bench.py --gpus N` with N above 1 exits with a message that says so."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def _layout_offset(list_block0, nb, Mp, b, lane, d):
    """Byte offset of dword d of point (block b, lane) of a list that starts at block
    list_block0 and has nb blocks, in the device layout of the codes as the interface documents
    it: lists padded to 64-point blocks of 64 * Mp bytes; within a list chunk-major, the 16-byte
    chunks first ([chunk][block][lane][16 B]), then the 4-byte chunks ([chunk][block][lane][4 B])."""
    base = list_block0 * 64 * Mp
    n16 = Mp // 16
    if d < 4 * n16:
        return base + ((d // 4) * nb + b) * 1024 + lane * 16 + (d % 4) * 4
    return base + n16 * nb * 1024 + ((d - 4 * n16) * nb + b) * 256 + lane * 4


@pytest.mark.parametrize("M,nlist,N", [(64, 16384, 100_000_000), (100, 1024, 1_000_000), (48, 1024, 1_000_000)])
def test_code_layout_offsets_stay_in_bounds_at_full_size(M, nlist, N):
    """The interleaved code layout at the size of the 100M-point configuration (6.4 GB: list
    bases and chunk offsets pass 2^32) and of the M = 100 one (4-byte tail chunks): the extreme
    addresses of every list -- first and last block, first and last lane, every dword -- are
    distinct per list, stay below the array's size, and an empty list's single read stays
    inside the 4 KiB of padding.  Also shows that 32-bit offset arithmetic would not do."""
    rng = np.random.default_rng(5)
    # list sizes with the imbalance of the trained index: some empty, some 4x the mean
    wts = rng.gamma(2.0, 1.0, nlist)
    wts[rng.choice(nlist, nlist // 64, replace=False)] = 0.0
    sizes = np.floor(wts / wts.sum() * N).astype(np.int64)
    sizes[np.argmax(sizes)] += N - sizes.sum()
    blocks = np.zeros(nlist + 1, dtype=np.int64)
    blocks[1:] = np.cumsum((sizes + 63) // 64)
    Mp = (M + 3) // 4 * 4
    code_bytes = int(blocks[-1]) * 64 * Mp
    top = 0
    for c in range(nlist):
        nb = int(blocks[c + 1] - blocks[c])
        b0 = int(blocks[c])
        if nb == 0:   # the scan reads one 1 KiB chunk at the list's base and ignores it
            assert b0 * 64 * Mp + 1024 <= code_bytes + 4096
            continue
        lo = _layout_offset(b0, nb, Mp, 0, 0, 0)
        hi = max(_layout_offset(b0, nb, Mp, nb - 1, 63, d) + 4 for d in range(Mp // 4))
        assert lo == b0 * 64 * Mp and hi == (b0 + nb) * 64 * Mp, (c, lo, hi)   # exactly the list's span
        top = max(top, hi)
    assert top == code_bytes
    if N >= 100_000_000:
        assert code_bytes > (1 << 32)
        assert (code_bytes & 0xFFFFFFFF) != code_bytes     # a 32-bit offset would wrap
    # inside one list: all (block, lane, dword) addresses distinct
    nb = 5
    seen = {_layout_offset(7, nb, Mp, b, l, d) for b in range(nb) for l in range(64) for d in range(Mp // 4)}
    assert len(seen) == nb * 64 * (Mp // 4) and min(seen) == 7 * 64 * Mp and max(seen) + 4 == (7 + nb) * 64 * Mp
