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
