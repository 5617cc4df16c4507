"""Host-only checks of the C ABI: the library loads without a GPU and exports every function the
public header declares; argument checks that need no device run here too."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "tandem.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tandem_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def binding():
    from paper_2402_08644_amd import binding as b

    if not os.path.exists(b.LIB_PATH):
        import __graft_entry__

        __graft_entry__.build()
    return b


def test_header_declares_the_four_entry_points():
    fns = header_functions()
    for name in ("tandem_project", "tandem_block_attn", "tandem_draft_attn", "tandem_decode_step"):
        assert name in fns


def test_library_exports_every_declared_function(binding):
    L = C.CDLL(binding.LIB_PATH)
    for name in header_functions():
        assert hasattr(L, name), f"{name} is declared in include/tandem.h but not exported"
    assert set(binding.EXPORTS) == set(header_functions())


def test_status_strings(binding):
    assert binding.status_string(binding.OK) == "ok"
    for code in range(1, 6):
        assert binding.status_string(code) not in ("ok", "unknown status")
    assert binding.status_string(99) == "unknown status"


def test_host_side_argument_checks_need_no_gpu(binding):
    L = binding.lib()
    d = binding.attn_desc(2, 4, 2, 128, 64, 4, 0.1, binding.BF16)
    # NULL pointers are rejected before anything touches a device
    assert L.tandem_draft_attn(C.byref(d), None, None, None, None, None, None, None, None, None, 0, None) == binding.ERR_NULL
    assert L.tandem_block_attn(C.byref(d), None, None, None, None, 4, None, None, 0, None) == binding.ERR_NULL
    assert L.tandem_block_attn(None, None, None, None, None, 4, None, None, 0, None) == binding.ERR_NULL
    bad = binding.attn_desc(2, 4, 3, 128, 64, 4, 0.1, binding.BF16)  # Hq not a multiple of Hkv
    assert binding.tandem_draft_attn_workspace(bad) == 0
    assert L.tandem_draft_attn(C.byref(bad), None, None, None, None, None, None, None, None, None, 0, None) == binding.ERR_SHAPE
    # workspace sizes are pure host functions of the shapes
    small = binding.attn_desc(64, 8, 8, 128, 256, 8, 0.1, binding.BF16)
    assert binding.tandem_draft_attn_workspace(small) == 0  # one split: no partials needed
    big = binding.attn_desc(8, 8, 8, 128, 2044, 4, 0.1, binding.BF16)
    assert binding.tandem_draft_attn_workspace(big) > 0
    assert binding.tandem_block_attn_workspace(big, 0) == 0 and binding.tandem_block_attn_workspace(big, 33) == 0
