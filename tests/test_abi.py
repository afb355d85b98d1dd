"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and the
calls that never touch the device (sizes, status strings, descriptor validation) behave."""
import ctypes
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


def declared_functions(header="ss.h"):
    text = (ROOT / "include" / header).read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ss_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2411_00288_amd as ss
    lib = ctypes.CDLL(str(ss.LIB_PATH))
    names = declared_functions()
    assert len(names) >= 9
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/ss.h but not exported"
    assert sorted(ss.EXPORTS) == names
    hooks = declared_functions("ss_debug.h")
    for n in hooks:
        assert hasattr(lib, n), f"{n} is declared in include/ss_debug.h but not exported"
    assert sorted(ss.DEBUG_EXPORTS) == hooks


def test_size_queries_and_descriptor_validation():
    import paper_2411_00288_amd as ss
    d = ss.make_desc(256, 256, 3, 3)
    assert ss.ss_packed_bytes(d) == 256 + 256 * 2304 + 256 * 2304 // 8       # 9/16 of dense + header
    assert ss.ss_dense_bytes(d) == 256 + 2 * 256 * 2304
    assert ss.ss_packed_bytes(ss.make_desc(40, 8, 3, 3)) == 256 + 2 * 3 * 1024 + 2 * 2 * 256
    assert ss.ss_conv2d_workspace_bytes(d, 32, 14, 14, (1, 1), (1, 1)) >= 0
    for bad, code in [(ss.make_desc(64, 3, 7, 7), ss.SS_ERR_UNSUPPORTED),       # K = 147
                      (ss.make_desc(0, 8, 1, 1), ss.SS_ERR_INVALID_ARG),
                      (ss.make_desc(8, 8, 1, 1, dtype=5), ss.SS_ERR_INVALID_ARG),
                      (ss.make_desc(8, 8, 1, 1, korder=2), ss.SS_ERR_INVALID_ARG)]:
        with pytest.raises(ss.SSError) as ei:
            ss.ss_packed_bytes(bad)
        assert ei.value.status == code
    assert ss.ss_dense_bytes(ss.make_desc(64, 3, 7, 7)) == 256 + 2 * 5 * 2048    # dense accepts any K
    assert "mask" in ss.ss_status_string(ss.SS_ERR_BAD_MASK)
    assert ss.ss_status_string(0) == "SS_OK"


def test_fusion_query_states_the_librarys_policy():
    import paper_2411_00288_amd as ss
    from paper_2411_00288_amd import workloads as wl
    d = lambda cout, cin, k, korder=wl.K_CRS, dtype=wl.BF16: ss.make_desc(cout, cin, k, k, dtype, korder)
    q = ss.ss_conv2d_pw_fused_query
    assert q(d(64, 64, 3), (1, 1), (1, 1), d(256, 64, 1), True) == (True, True)        # stage-1 bottleneck
    assert q(d(128, 128, 3), (2, 2), (1, 1), d(512, 128, 1), True) == (True, True)
    assert q(d(256, 256, 3), (1, 1), (1, 1), d(1024, 256, 1), True) == (True, False)   # supported, but two calls are faster
    assert q(d(128, 128, 3), (1, 1), (1, 1), d(512, 128, 1), False) == (True, False)   # dense twin: up to 64 wide
    assert q(d(64, 64, 3), (1, 1), (1, 1), d(256, 64, 1), False) == (True, True)
    assert q(d(512, 512, 3), (1, 1), (1, 1), d(2048, 512, 1), True) == (False, False)  # wider than a tile
    assert q(d(64, 24, 3), (1, 1), (1, 1), d(256, 64, 1), True) == (False, False)      # no fast staging for the first layer
    assert q(d(64, 24, 3, wl.K_RSC), (1, 1), (1, 1), d(256, 64, 1), True) == (True, True)
    assert q(d(384, 96, 1), (1, 1), (0, 0), d(96, 384, 1), True) == (True, True)       # ConvNeXt block
    assert q(d(384, 96, 1), (2, 2), (0, 0), d(96, 384, 1), True) == (False, False)
    assert q(d(384, 160, 1), (1, 1), (0, 0), d(96, 384, 1), True) == (False, False)    # cin > 128
    assert q(d(64, 64, 3, dtype=wl.I8), (1, 1), (1, 1), d(256, 64, 1, dtype=wl.I8), True) == (False, False)
    with pytest.raises(ss.SSError) as e:
        q(d(64, 64, 3), (1, 1), (1, 1), d(256, 32, 1), True)                           # second layer on other channels
    assert e.value.status == ss.SS_ERR_INVALID_ARG
