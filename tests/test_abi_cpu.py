"""CPU-only checks of the boundary: the shared library loads, exports every symbol the header
declares, and rejects bad arguments on the host before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2601_10639_amd import stemlib as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(L.LIB_PATH):
        from paper_2601_10639_amd import build
        build.build()
    return L.lib()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "stem.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(stem_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    declared = _declared_symbols()
    assert len(declared) >= 10
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in stem.h but not exported by libstem.so"
    assert sorted(L.SYMBOLS) == declared
    for name in ("stem_create", "stem_destroy", "stem_ffn_forward", "stem_ffn_backward", "stem_embed_grad",
                 "stem_embed_sparse_adamw", "stem_prefetch_rows", "stem_sync_status"):
        assert callable(getattr(L, name))


def test_status_strings(lib):
    names = [L.status_string(i) for i in range(7)]
    assert names == ["STEM_OK", "STEM_ERR_INVALID_ARG", "STEM_ERR_SHAPE", "STEM_ERR_ID_RANGE",
                     "STEM_ERR_WORKSPACE", "STEM_ERR_UNSUPPORTED", "STEM_ERR_HIP"]
    assert lib.stem_profile_kernels() >= 10


def test_create_rejects_bad_descriptors_on_the_host(lib):
    out = ctypes.c_void_p(123)

    def create(d, F, V, dt, T):
        desc = L.stem_layer_desc(d, F, V, dt)
        return lib.stem_create(ctypes.byref(out), ctypes.byref(desc), T, 0)

    assert create(100, 256, 10, L.STEM_BF16, 8) == L.STEM_ERR_UNSUPPORTED   # d_model not a multiple of 64
    assert out.value is None
    assert b"multiples of 64" in lib.stem_last_error(None)
    assert create(64, 64, 10, 7, 8) == L.STEM_ERR_INVALID_ARG               # unknown dtype
    assert create(64, 64, 0, L.STEM_BF16, 8) == L.STEM_ERR_SHAPE            # empty vocabulary
    assert create(64, 64, 10, L.STEM_BF16, -1) == L.STEM_ERR_SHAPE          # negative capacity
    assert create(6, 8, 10, L.STEM_F32, 8) == L.STEM_ERR_UNSUPPORTED        # fp32 needs multiples of 4
    assert lib.stem_create(None, None, 8, 0) == L.STEM_ERR_INVALID_ARG
    # bf16 activations of 2 GiB or more do not fit the kernels' 32-bit buffer offsets: refused with the limit named
    assert create(2048, 8192, 128256, L.STEM_BF16, 131072) == L.STEM_ERR_SHAPE
    assert b"2^31" in lib.stem_last_error(None)
    assert create(8192, 2048, 1000, L.STEM_BF16, 131072) == L.STEM_ERR_SHAPE      # [T, d_model] is the large one here
    assert create(32768, 32768, 10, L.STEM_BF16, 8) == L.STEM_ERR_SHAPE           # fp32 weight gradient of 4 GiB


def test_null_context_is_refused(lib):
    z = ctypes.c_void_p(None)
    assert lib.stem_ffn_forward(z, z, z, z, z, z, 1, 1, z, z, z, z, z) == L.STEM_ERR_INVALID_ARG
    assert lib.stem_ffn_backward(z, z, z, z, z, z, z, 1, z, z, 1, z, z, z, z, 0, z) == L.STEM_ERR_INVALID_ARG
    assert lib.stem_embed_grad(z, z, z, 1, z, z, z, z, z, z, z) == L.STEM_ERR_INVALID_ARG
    assert lib.stem_embed_sparse_adamw(z, z, z, 1, z, z, z, z, z, None, z) == L.STEM_ERR_INVALID_ARG
    assert lib.stem_sync_status(z, z) == L.STEM_ERR_INVALID_ARG
    assert lib.stem_profile_enable(z, 1) == L.STEM_ERR_INVALID_ARG
    assert lib.stem_reserve(z, 1) == L.STEM_ERR_INVALID_ARG
    assert lib.stem_set_prefetch_mode(z, 0) == L.STEM_ERR_INVALID_ARG
    assert lib.stem_ffn_forward_residual(z, z, z, z, z, z, 1, 1, z, z, z) == L.STEM_ERR_INVALID_ARG
    assert lib.stem_embed_grad_presorted(z, z, 1, z, z, z, z) == L.STEM_ERR_INVALID_ARG
    # the calls that need no context check their arguments on the host as well
    assert lib.stem_embed_grad_noalloc(7, 10, 8, z, z, 1, z, z, z, z, z, z, z, z) == L.STEM_ERR_INVALID_ARG
    assert lib.stem_embed_grad_noalloc(L.STEM_BF16, 10, 8, z, z, L.STEM_NOALLOC_MAX_TOKENS + 1, z, z, z, z, z, z, z, z) == L.STEM_ERR_SHAPE
    assert b"65536" in lib.stem_last_error(None)
    assert lib.stem_measure_peak(9, z, z, 4096, 1, z, None) == L.STEM_ERR_INVALID_ARG
    lib.stem_destroy(z)  # allowed


def test_binding_refuses_wrong_dtypes_before_calling():
    import torch

    class Fake:
        handle = ctypes.c_void_p(None)
        torch_dtype = torch.bfloat16

    x = torch.zeros(4, 64, dtype=torch.float32)
    with pytest.raises(TypeError):
        L.stem_ffn_forward(Fake(), x, torch.zeros(4, dtype=torch.int32), x, x, x, x)


def test_early_touch_of_gathered_rows_stays_inside_the_table():
    """The gate product touches, a few K tiles before its epilogue, the two 128-byte lines of the table
    row that a wavefront's 128 output columns will read.  Host-side model of those addresses (column
    of the wavefront's quadrant, second line only if the row is that wide) over every d_ff the bf16
    path accepts up to 1024 and the first and last table rows: each 4-byte touch lies inside the row."""
    for F in range(64, 1025, 64):
        ntn = (F + 255) // 256
        for tn in range(ntn):
            for wn in (0, 1):
                ncol = tn * 256 + wn * 128
                col = ncol if ncol < F else 0
                second = col + 64 if col + 64 < F else col
                for first_elem in (col, second):
                    assert 0 <= first_elem and first_elem * 2 + 4 <= F * 2, (F, tn, wn, first_elem)


def test_tile_map_model_covers_every_tile_once():
    """The large GEMM maps workgroup ids to output tiles in XCD-major runs walked in bands of tile rows
    (4, or 7 in the dH product).  Host-side model of that map over ragged and full grids, incl. fewer
    workgroups than XCDs and band heights that do not divide the number of tile rows: every tile is
    produced by exactly one workgroup."""
    def tile_of_block(b, nb, ntm, ntn, gm):
        q, r = nb >> 3, nb & 7
        xcd, idx = b & 7, b >> 3
        lin = xcd * q + min(xcd, r) + idx
        per_group = gm * ntn
        group = lin // per_group
        first = group * gm
        gsize = min(ntm - first, gm)
        inside = lin - group * per_group
        return first + inside % gsize, inside // gsize

    for gm in (4, 7):
        for ntm in (1, 2, 3, 5, 7, 8, 9, 13, 64):
            for ntn in (1, 2, 3, 8, 31, 32):
                nb = ntm * ntn
                seen = set()
                for b in range(nb):
                    tm, tn = tile_of_block(b, nb, ntm, ntn, gm)
                    assert 0 <= tm < ntm and 0 <= tn < ntn, (gm, ntm, ntn, b, tm, tn)
                    seen.add((tm, tn))
                assert len(seen) == nb, (gm, ntm, ntn)
