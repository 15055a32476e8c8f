"""The C-ABI library loads and exports every symbol that include/attncache.h declares.
No compute call is made here (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "attncache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(?:int32_t|const char \*|size_t)\s*\*?\s*(att\w+)\s*\(", text)
    return sorted(set(names))


def test_header_declares_the_four_entry_points():
    names = _declared_symbols()
    for n in ("attncache_build_db", "attncache_search", "attncache_apply", "attention_exact"):
        assert n in names


def test_library_exports_every_declared_symbol():
    from paper_2510_25979_amd import binding, build
    if build.stale():
        build.build(force=True)
    lib = ctypes.CDLL(binding.lib_path())
    for n in _declared_symbols():
        assert hasattr(lib, n), n
    assert sorted(binding.SYMBOLS) == _declared_symbols()


def test_status_strings_and_version():
    from paper_2510_25979_amd import binding
    L = binding.lib()
    assert L.attncache_version() >= 1000
    assert L.attncache_status_string(0) == b"ok"
    for code in range(-10, 0):
        assert L.attncache_status_string(code) != b"unknown status"
    assert L.attncache_status_string(-99) == b"unknown status"


def test_workspace_query_validates_without_a_gpu():
    from paper_2510_25979_amd import binding
    d = binding.DbDesc(n_emb=1000, emb_dim=256, emb_dtype=binding.AC_F16, metric=binding.AC_IP,
                       n_entries=1000, n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=64,
                       seq_len=128, map_dtype=binding.AC_BF16, causal=1, maps_on_host=0, map_layout=0)
    assert binding.attncache_workspace_bytes(d, 64, 1) > 0
    assert binding.attncache_workspace_bytes(d, 64, 4) > binding.attncache_workspace_bytes(d, 64, 1)
    import pytest
    with pytest.raises(binding.AttnCacheError) as e:
        binding.attncache_workspace_bytes(d, 64, 65)
    assert e.value.status == -5
    assert binding.attncache_map_entry_bytes(d) == 2 * 4 * 128 * 128 * 2
    d.map_layout = binding.AC_LAYOUT_PACKED
    assert binding.attncache_map_entry_bytes(d) == 2 * 4 * 20 * 512 * 2      # 20 KiB per head
    assert binding.packed_tile_elems(1024, True) == 32 * 33 * 512
    assert binding.packed_tile_elems(96, False) == 96 * 96
    d.seq_len = 100
    with pytest.raises(binding.AttnCacheError) as e:
        binding.attncache_workspace_bytes(d, 64, 1)
    assert e.value.status == -2
    d.seq_len, d.n_kv_heads = 128, 3
    with pytest.raises(binding.AttnCacheError):
        binding.attncache_workspace_bytes(d, 64, 1)


def test_workspace_sizes_follow_the_search_plan():
    """Workspace = one (score, row) pair per query and group (padded to 256 bytes) + k groups of
    candidate scores per query for k > 1 + 256 bytes; the group size depends on the path the
    shape takes.  Pure host logic."""
    from paper_2510_25979_amd import binding

    def ws(N, E, B, k, dtype=None, metric=None):
        d = binding.DbDesc(n_emb=N, emb_dim=E, emb_dtype=binding.AC_F16 if dtype is None else dtype,
                           metric=binding.AC_IP if metric is None else metric,
                           n_entries=N, n_layers=1, n_q_heads=1, n_kv_heads=1, head_dim=64,
                           seq_len=32, map_dtype=binding.AC_BF16, causal=1, maps_on_host=0, map_layout=0)
        return binding.attncache_workspace_bytes(d, B, k)

    def expect(B, G, k, rpw):
        part = (B * G * 8 + 255) // 256 * 256
        return part + (B * k * rpw * 4 if k > 1 else 0) + 256

    # The size is the larger of what the inner-product and the L2 path of the shape need (the
    # metric is a property of the handle, not of the query): the vector-ALU path has groups of
    # 256 rows.
    def both(B, N, k, rpw_ip):
        return max(expect(B, -(-N // rpw_ip), k, rpw_ip), expect(B, -(-N // 256), k, 256))

    # matrix-core path, top-1, small database: one group per 128-row workgroup
    assert ws(10000, 256, 64, 1) == both(64, 10000, 1, 128)
    # matrix-core path, top-k, small database: groups of 32 rows (the long-sequence workload's search)
    assert ws(1024, 512, 16, 4) == both(16, 1024, 4, 32)
    assert ws(32768, 128, 9, 5) == both(9, 32768, 5, 32)
    # just above the limit of the small-group plan: back to one group per workgroup
    assert ws(40000, 256, 10, 3) == both(10, 40000, 3, 128)
    # million-row index: ~480 groups of a multiple of 64 rows
    rpw = 64 * -(-1000000 // (64 * 480))
    assert ws(1000000, 256, 256, 1) == both(256, 1000000, 1, rpw)
    # fp32 features: vector-ALU path only
    assert ws(1024, 128, 4, 3, dtype=binding.AC_F32) == expect(4, 4, 3, 256)
    # monotone in the batch
    assert ws(10000, 256, 128, 1) > ws(10000, 256, 64, 1)


def test_product_path_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2510_25979_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src, f
                assert "liboracle" not in src and "attncache_oracle" not in src, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            src = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2510_25979_amd" not in src and "libattncache" not in src, f


def test_header_is_plain_c(tmp_path):
    """The boundary must be usable from C: the header compiles as C99 with warnings as errors,
    and a C translation unit can take the address of every declared entry point."""
    import subprocess
    names = _declared_symbols()
    src = tmp_path / "use_abi.c"
    body = "\n".join(f"  table[{i}] = (void (*)(void))&{n};" for i, n in enumerate(names))
    src.write_text('#include "attncache.h"\n'
                   f"void (*table[{len(names)}])(void);\n"
                   "void fill(void) {\n" + body + "\n}\n"
                   "int main(void) { attncache_db_desc d; (void)d; fill(); return AC_OK; }\n")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-c",
                    "-I", os.path.join(ROOT, "include"), str(src), "-o", str(tmp_path / "use_abi.o")],
                   check=True)
