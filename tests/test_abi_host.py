"""Host-side checks that need no GPU: the library loads, exports every declared symbol, sizes
and the pool allocator behave as include/relaygr.h says (CPU only; no compute call is made)."""
import ctypes as C
import os
import re

import pytest

import paper_2601_01712_amd as rg
from paper_2601_01712_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = rg.load_library()
    header = open(os.path.join(ROOT, "include", "relaygr.h")).read()
    declared = set(re.findall(r"\b(relaygr_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(rg.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_kv_footprint_matches_papers_table():
    rows = [ln.split() for ln in open(os.path.join(ROOT, "tests", "golden", "kv_cache_size.txt"))
            if ln.strip() and not ln.startswith("#")]
    for L, nl, d, e, want in rows:
        heads = int(d) // 64
        cfg = rg.make_config(int(nl), int(d), heads, "fp32" if int(e) == 4 else "bf16")
        assert rg.relaygr_kv_footprint_bytes(cfg, int(L)) == int(want)
    cfg = rg.make_config(8, 512, 8, "bf16")
    assert rg.relaygr_kv_footprint_bytes(cfg, 8192) == 134217728
    assert rg.relaygr_kv_pool_bytes_for(cfg, 8192, 256) == 134217728
    assert rg.relaygr_kv_pool_bytes_for(cfg, 8193, 256) == 134217728 + 256 * 16384
    # the two 16-bit storage types take the same space and scratch
    half = rg.make_config(8, 512, 8, "fp16")
    assert rg.relaygr_kv_footprint_bytes(half, 8192) == 134217728
    assert rg.relaygr_scratch_bytes(half, 16, 65536, 8192) == rg.relaygr_scratch_bytes(cfg, 16, 65536, 8192) > 0


@pytest.mark.parametrize("bad", [
    dict(n_layers=0), dict(d_model=96), dict(n_heads=3), dict(d_model=512, n_heads=2),
    dict(dtype="bf16", d_model=64, n_heads=2), dict(dtype="fp16", d_model=64, n_heads=2), dict(ln_eps=0.0),
])
def test_unsupported_configs_are_rejected(bad):
    kw = dict(n_layers=2, d_model=256, n_heads=4, dtype="bf16", ln_eps=1e-5)
    kw.update(bad)
    cfg = rg.make_config(**kw)
    assert rg.relaygr_kv_footprint_bytes(cfg, 100) == 0
    assert rg.relaygr_scratch_bytes(cfg, 1, 100, 100) == 0


def test_scratch_bytes_grows_with_the_call_size():
    cfg = rg.make_config(8, 512, 8, "bf16")
    a = rg.relaygr_scratch_bytes(cfg, 16, 0, 8192)
    b = rg.relaygr_scratch_bytes(cfg, 16, 65536, 8192)
    assert 0 < a < b
    assert rg.relaygr_scratch_bytes(cfg, 0, 0, 10) == 0


class FakeSlabPool:
    """A pool over an address range that is never dereferenced (the allocator is host-only)."""

    def __init__(self, cfg, pages, page_tokens=256):
        lib = rg.load_library()
        page_bytes = rg.relaygr_kv_pool_bytes_for(cfg, page_tokens, page_tokens)
        self.handle = C.c_void_p()
        rc = lib.relaygr_kv_pool_create(C.byref(cfg), C.c_void_p(0x10000000), pages * page_bytes + 17, page_tokens,
                                        C.byref(self.handle))
        assert rc == 0, rg.relaygr_last_error()

    def __del__(self):
        rg.load_library().relaygr_kv_pool_destroy(self.handle)


def test_pool_alloc_free_lookup_and_stale_handles():
    cfg = rg.make_config(4, 256, 4, "bf16")
    p = FakeSlabPool(cfg, pages=10)
    st = rg.relaygr_kv_pool_stats(p)
    assert st == {"pages_total": 10, "pages_free": 10, "live_entries": 0, "largest_free_extent": 10}
    h1 = rg.relaygr_kv_pool_alloc(p, 111, 700)      # 3 pages
    h2 = rg.relaygr_kv_pool_alloc(p, 222, 256)      # 1 page
    h3 = rg.relaygr_kv_pool_alloc(p, 333, 1025)     # 5 pages
    assert len({h1, h2, h3}) == 3 and 0 not in (h1, h2, h3)
    assert rg.relaygr_kv_pool_stats(p)["pages_free"] == 1
    assert rg.relaygr_kv_pool_lookup(p, 222) == h2
    assert rg.relaygr_kv_pool_lookup(p, 999) == rg.RELAYGR_NO_CACHE
    assert rg.relaygr_kv_pool_entry_len(p, h3) == 1025
    # a second live entry for the same user is refused
    with pytest.raises(rg.RelayGRError) as e:
        rg.relaygr_kv_pool_alloc(p, 111, 10)
    assert e.value.code == rg.RELAYGR_EINVAL
    # no extent of 2 pages is left: the pool says so instead of evicting a live entry
    with pytest.raises(rg.RelayGRError) as e:
        rg.relaygr_kv_pool_alloc(p, 444, 300)
    assert e.value.code == rg.RELAYGR_ENOSPC
    assert "no free extent" in str(e.value)
    assert rg.relaygr_kv_pool_lookup(p, 111) == h1   # still live
    # free the middle entry, then the first: the two holes coalesce into one extent of 4 pages
    rg.relaygr_kv_pool_free(p, h2)
    rg.relaygr_kv_pool_free(p, h1)
    st = rg.relaygr_kv_pool_stats(p)
    assert st["pages_free"] == 5 and st["largest_free_extent"] == 4 and st["live_entries"] == 1
    # stale handles are rejected everywhere
    for fn in (lambda: rg.relaygr_kv_pool_free(p, h1), lambda: rg.relaygr_kv_pool_entry_len(p, h2),
               lambda: rg.relaygr_kv_pool_free(p, 0), lambda: rg.relaygr_kv_pool_free(p, 12345 << 32 | 77)):
        with pytest.raises(rg.RelayGRError) as e:
            fn()
        assert e.value.code == rg.RELAYGR_ENOENT
    # the slot is reused with a new generation: the old handle stays stale
    h4 = rg.relaygr_kv_pool_alloc(p, 111, 1000)     # 4 pages, fits the coalesced hole
    assert h4 != h1 and rg.relaygr_kv_pool_lookup(p, 111) == h4
    with pytest.raises(rg.RelayGRError):
        rg.relaygr_kv_pool_entry_len(p, h1)
    rg.relaygr_kv_pool_free(p, h3)
    rg.relaygr_kv_pool_free(p, h4)
    st = rg.relaygr_kv_pool_stats(p)
    assert st["pages_free"] == 10 and st["largest_free_extent"] == 10 and st["live_entries"] == 0


def test_pool_locate_follows_the_documented_tile_layout():
    cfg = rg.make_config(2, 128, 2, "bf16")   # d_head 64
    p = FakeSlabPool(cfg, pages=4, page_tokens=128)
    h0 = rg.relaygr_kv_pool_alloc(p, 1, 100)  # page 0
    h = rg.relaygr_kv_pool_alloc(p, 2, 200)   # pages 1-2 -> first tile index 2
    tile_stride = 2 * 2 * 64 * 128            # layers * (K,V) * 64 tokens * d
    layer_stride = 2 * 64 * 128
    k, v = rg.relaygr_kv_pool_locate(p, h, 1, 70, 64 + 5)    # layer 1, token 70 -> tile 1, r 6; head 1, f 5
    base = (2 + 1) * tile_stride + 1 * layer_stride + 1 * 2 * 64 * 64
    # bf16 tiles are stored in MFMA fragment order: 1 KiB fragments of 64 lanes x 8 elements.
    # K: token 6 -> key block 0, lane 6; feature 5 -> k-step 0, half 0, element 5
    assert k == base + ((0 * 4 + 0) * 64 + 0 * 32 + 6) * 8 + 5
    # V: feature 5 -> feature block 0, lane 5; token 6 -> key block 0, step 0, half 1 (tokens 4..7), slot 2
    assert v == base + 64 * 64 + (((0 * 2 + 0) * 2 + 0) * 64 + 1 * 32 + 5) * 8 + 2
    # the fp32 layout is plain: K [token][feature], V [feature][token]
    cfg32 = rg.make_config(2, 128, 2, "fp32")
    p32 = FakeSlabPool(cfg32, pages=4, page_tokens=128)
    h32 = rg.relaygr_kv_pool_alloc(p32, 2, 200)
    k32, v32 = rg.relaygr_kv_pool_locate(p32, h32, 1, 70, 64 + 5)
    base32 = 1 * tile_stride + 1 * layer_stride + 1 * 2 * 64 * 64
    assert k32 == base32 + 6 * 64 + 5 and v32 == base32 + 64 * 64 + 5 * 64 + 6
    seen = set()
    for tok in (0, 63, 64, 199):
        for feat in (0, 63, 64, 127):
            for layer in (0, 1):
                kk, vv = rg.relaygr_kv_pool_locate(p, h, layer, tok, feat)
                assert kk not in seen and vv not in seen
                seen.update((kk, vv))
                assert 2 * tile_stride <= kk < 6 * tile_stride and 2 * tile_stride <= vv < 6 * tile_stride
    with pytest.raises(rg.RelayGRError):
        rg.relaygr_kv_pool_locate(p, h, 0, 200, 0)
    del h0


def test_pool_create_validates_arguments():
    lib = rg.load_library()
    cfg = rg.make_config(2, 128, 2, "bf16")
    out = C.c_void_p()
    assert lib.relaygr_kv_pool_create(C.byref(cfg), C.c_void_p(0x1000), 1 << 30, 100, C.byref(out)) == rg.RELAYGR_EINVAL
    assert lib.relaygr_kv_pool_create(C.byref(cfg), C.c_void_p(0x1001), 1 << 30, 128, C.byref(out)) == rg.RELAYGR_EINVAL
    assert lib.relaygr_kv_pool_create(C.byref(cfg), C.c_void_p(0x1000), 1000, 128, C.byref(out)) == rg.RELAYGR_ENOSPC
    assert "smaller than one page" in rg.relaygr_last_error()


def test_attention_form_setter_rejects_a_null_context():
    lib = rg.load_library()
    assert lib.relaygr_ctx_set_attention(None, B.ATTENTION_FORMS["softmax"]) == rg.RELAYGR_EINVAL
    assert "null context" in rg.relaygr_last_error()
    assert B.ATTENTION_FORMS == {"silu": 0, "softmax": 1}       # RELAYGR_ATTN_SILU, RELAYGR_ATTN_SOFTMAX
    header = open(os.path.join(ROOT, "include", "relaygr.h")).read()
    assert re.search(r"#define\s+RELAYGR_ATTN_SILU\s+0", header) and re.search(r"#define\s+RELAYGR_ATTN_SOFTMAX\s+1", header)


def test_header_is_valid_c99_and_links_against_the_library(tmp_path):
    """The boundary is a C ABI: a C99 translation unit that includes the header, takes the address of
    every declared function and calls the host-only ones must compile without warnings and link."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    header = open(os.path.join(ROOT, "include", "relaygr.h")).read()
    names = sorted(set(re.findall(r"\b(relaygr_[a-z_0-9]+)\s*\(", header)))
    src = tmp_path / "abi.c"
    src.write_text(
        '#include "relaygr.h"\n#include <stdio.h>\n'
        "typedef void (*fn)(void);\n"
        "int main(void) {\n"
        "  fn table[] = {" + ", ".join(f"(fn){n}" for n in names) + "};\n"
        "  relaygr_model_config cfg = {8, 256, 8, RELAYGR_DTYPE_FP32, 1e-5f};\n"
        "  size_t kv = relaygr_kv_footprint_bytes(&cfg, 2048);\n"
        "  int rc = relaygr_ctx_set_attention(NULL, RELAYGR_ATTN_SOFTMAX);\n"
        '  printf("%zu %d %zu\\n", kv, rc, sizeof(table) / sizeof(table[0]));\n'
        "  return 0;\n}\n")
    rg.load_library()
    from paper_2601_01712_amd import build as _build
    lib_dir = os.path.dirname(_build.LIB)
    exe = tmp_path / "abi"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", lib_dir, "-lrelaygr", f"-Wl,-rpath,{lib_dir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == 32 * 1024 * 1024          # the paper's example: 2K tokens, 8 layers, d 256, fp32 (Section 4.1)
    assert int(out[1]) == rg.RELAYGR_EINVAL
    assert int(out[2]) == len(names) == len(rg.EXPORTS)
