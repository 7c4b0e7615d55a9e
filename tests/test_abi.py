"""The C-ABI library loads and exports every symbol include/rov.h declares (no GPU needed)."""
import ctypes
import os
import re

from paper_2410_07531_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "rov.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rov_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    names = _declared()
    assert "rov_dropout_mask_generate" in names and "rov_gemm" in names
    assert os.path.exists(binding.LIB_PATH), "build the library first (__graft_entry__.build())"
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), "librov.so does not export %s" % n
    assert sorted(binding.SIGNATURES) == names


def test_host_only_entry_points():
    L = binding.load()
    assert L.rov_version().startswith(b"rov")
    assert binding.mask_words(1, 2, 128) == 2 * 4 * 4 * 16
    assert binding.mask_words(1, 1, 70) == 3 * 3 * 16
    assert binding.mask_words(0, 1, 70) == 0
    assert binding.mask_philox_calls(1, 2, 128) == 64 * 128
    assert binding.mask_philox_calls(1, 1, 70) == 64 * 36
    assert binding.mask_philox_calls(1, 1, 1) == 64 * 4
    assert binding.mask_shape(2, 3, 70) == (2, 3, 3, 3, 16)
    assert L.rov_last_hip_error() == 0


def test_gemm_tile_width_rule():
    # host logic: the width that leaves least of the last round of workgroups empty (256 compute
    # units), widest on ties; the limiter model's copy of the rule must agree with the library's
    from paper_2410_07531_amd import limiter_model as LM
    assert binding.gemm_tile_cols(2048, 14336) == 224      # 448 tiles of 256 -> 512 tiles of 224: two full rounds
    assert binding.gemm_tile_cols(2048, 6144) == 192       # 192 tiles -> 256 tiles: one full round
    assert binding.gemm_tile_cols(2048, 4096) == 128
    assert binding.gemm_tile_cols(8192, 8192) == 256 and binding.gemm_tile_cols(16384, 14336) == 256
    assert binding.gemm_tile_cols(1, 4) == 128             # one tile either way: the narrowest is the cheapest
    for M in (1, 256, 300, 2048, 4096, 8192, 16384):
        for N in range(4, 20000, 364):
            assert binding.gemm_tile_cols(M, N) == LM.gemm_tile_cols(LM.MI355X, M, N), (M, N)
    L = binding.load()
    assert L.rov_gemm_tile_cols(0, 8) == binding.ERR_INVALID and L.rov_gemm_tile_cols(8, -1) == binding.ERR_INVALID
    prev = binding.set_gemm_tile_cols(160)
    try:
        assert binding.gemm_tile_cols(8192, 8192) == 160
    finally:
        binding.set_gemm_tile_cols(prev)
    assert binding.gemm_tile_cols(8192, 8192) == 256


def test_no_oracle_on_the_product_path():
    # the package must never import the oracle (and the oracle never the package)
    pkg = os.path.join(ROOT, "paper_2410_07531_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", src, flags=re.M), f
                assert "liboracle" not in src and "philox_oracle" not in src, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            src = open(os.path.join(ROOT, "oracle", f)).read()
            assert not re.search(r"^\s*(from|import)\s+paper_2410_07531_amd\b", src, flags=re.M), f
            assert "librov" not in src, f
