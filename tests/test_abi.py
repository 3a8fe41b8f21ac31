"""The C-ABI library loads and exports every entry point the header declares
(no compute calls: runs without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "tier.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tier_[a-z_]+)\s*\(", text)))


def _lib_path():
    from paper_2111_05894_amd import tier
    if not os.path.exists(tier.LIB_PATH):
        from paper_2111_05894_amd import build
        build.build()
    return tier.LIB_PATH


def test_header_names_match_binding():
    from paper_2111_05894_amd import tier
    assert _declared() == sorted(tier.EXPORTS)


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(_lib_path())
    for name in _declared():
        assert hasattr(lib, name), name


def test_host_only_entry_points():
    from paper_2111_05894_amd import tier
    from oracle import oracle as orc
    _lib_path()
    # bounds are pure host arithmetic
    cn, ce = tier.tier_blocks_bounds(10**6, 1024, (15, 10, 5))
    assert cn == [1024, 16384, 180224, 1000000] and ce == [15360, 163840, 901120]
    assert (cn, ce) == tuple(orc.frontier_bounds(1024, (15, 10, 5), 10**6))
    with pytest.raises(tier.TierError):
        tier.tier_blocks_bounds(100, 10, (0,))
    with pytest.raises(tier.TierError):
        tier.tier_blocks_bounds(100, 10, (65,))
    with pytest.raises(tier.TierError):
        tier.tier_blocks_bounds(100, 10, (1,) * 9)
    # mini-batch seeds: both sides implement the same counter-based generator
    for s, e, b in ((0, 0, 0), (5894, 0, 7), (2**64 - 1, 3, 2**31), (0x0123456789ABCDEF, 11, 187)):
        assert tier.tier_batch_seed(s, e, b) == orc.batch_seed(s, e, b)
    assert tier._load().tier_strerror(-4).decode().startswith("output buffer")


def test_missing_library_raises(tmp_path, monkeypatch):
    from paper_2111_05894_amd import tier
    monkeypatch.setattr(tier, "_lib", None)
    monkeypatch.setattr(tier, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        tier._load()


def test_header_is_plain_c(tmp_path):
    """The boundary is a C header: it compiles as C11 on its own (no HIP, no C++, no torch)."""
    import subprocess
    src = tmp_path / "use_tier.c"
    src.write_text('#include "tier.h"\n'
                   "int probe(void) { tier_gather_stats s; tier_csr g; tier_feat f; (void)s; (void)g; (void)f;\n"
                   "  return TIER_OK + TIER_MAX_LAYERS + TIER_MAX_FANOUT + TIER_MAX_BATCHES + (int)sizeof(tier_blocks_batch); }\n")
    r = subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
