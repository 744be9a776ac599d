"""CPU-only checks of the boundary: the library loads and exports every symbol that
include/moe.h declares, and host-side validation rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

from paper_2605_11005_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header="moe.h"):
    src = open(os.path.join(ROOT, "include", header)).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.lib_path()):
        import __graft_entry__ as g
        g.build()
    return B.load_library()


def test_header_declares_the_five_calls():
    names = _declared()
    for n in ("moe_route", "moe_dispatch", "moe_expert_fwd", "moe_expert_bwd", "moe_combine"):
        assert n in names


def test_every_declared_symbol_is_exported(lib):
    for n in _declared():
        assert hasattr(lib, n), n
    assert set(_declared()) == set(B.EXPORTS)
    from paper_2605_11005_amd import alloc as A
    alloc_names = [n for n in _declared("moe_alloc.h") if n != "moe_alloc_profile_fn"]
    for n in alloc_names:
        assert hasattr(lib, n), n
    assert set(alloc_names) == set(A.EXPORTS)


def test_error_strings_and_workspace_sizes(lib):
    assert lib.moe_error_string(0) == b"ok"
    for c in (1, 2, 3, 4, 99):
        assert len(lib.moe_error_string(c)) > 0
    # a [cap,f] bf16 for the forward, three such for the backward
    assert B.moe_workspace_bytes(B.WS_EXPERT_FWD, B.MOE_BF16, 0, 0, 64, 128, 4, 1000) >= 1000 * 128 * 2
    assert B.moe_workspace_bytes(B.WS_EXPERT_BWD, B.MOE_BF16, 0, 0, 64, 128, 4, 1000) >= 3 * 1000 * 128 * 2
    assert B.moe_workspace_bytes(B.WS_DISPATCH, B.MOE_BF16, 1024, 8, 64, 128, 4, 1000) >= 16 * 4 * 4


def test_router_workspace_reflects_how_the_router_gemms_are_cut(lib):
    """The router workspace is the larger of what the forward (fp32 logits per range of a cut
    contraction) and the backward (dlogits as bf16 + fp32 chunk sums of dWr) need; its size shows
    the cuts the host chose.  Counted for 256 CUs (what a host without a GPU assumes, and what the
    chip has): rounds of the CUs x (k-tiles per work item + 16)."""
    al = lambda v: (v + 255) // 256 * 256
    ws = lambda T, d, E: B.moe_workspace_bytes(B.WS_ROUTER, B.MOE_BF16, T, 8, d, 2048, E, 0)
    # T = 32768, d = 7168, E = 256: 128 logit tiles -> two ranges of d (one round); 28 dWr tiles -> 9 token
    # chunks (252 work items, one round; 10 chunks would take two rounds)
    T, d, E = 32768, 7168, 256
    assert ws(T, d, E) == 256 + max(al(T * E * 2) + al(9 * d * E * 4), al(2 * T * E * 4))
    # 65536 tokens: 256 logit tiles fill the chip, the contraction stays whole; dWr as before
    T = 65536
    assert ws(T, d, E) == 256 + al(T * E * 2) + al(9 * d * E * 4)
    # a short contraction (four pairs of k-tiles) is never cut; 1 x 1 dWr tile over 2048 tokens: at least four
    # k-tiles per chunk bounds the chunks at 16
    T, d, E = 2048, 256, 128
    assert ws(T, d, E) == 256 + al(T * E * 2) + al(16 * d * E * 4)
    # 23 pairs of k-tiles, 128 logit tiles: two ranges (12 and 11 pairs; three would need a second round);
    # 6 dWr tiles: 32 token chunks (the most allowed) still fit one round
    T, d, E = 32768, 1472, 256
    assert ws(T, d, E) == 256 + max(al(T * E * 2) + al(32 * d * E * 4), al(2 * T * E * 4))
    assert al(2 * T * E * 4) > al(T * E * 2) + al(32 * d * E * 4)          # (the forward's need decides here)


def test_host_validation_rejects_before_launch(lib):
    """Only calls that fail validation are made here (no GPU needed: nothing is launched)."""
    P = ctypes.c_void_p
    fake = P(4096)
    # k > E, bad slice, unknown gate mode, NULL pointers
    assert lib.moe_route(fake, 4, 8, 9, 0, 0, 8, fake, fake, fake, None) == 1
    assert lib.moe_route(fake, 4, 8, 2, 0, 4, 8, fake, fake, fake, None) == 1
    assert lib.moe_route(fake, 4, 8, 2, 7, 0, 8, fake, fake, fake, None) == 1
    assert lib.moe_route(None, 4, 8, 2, 0, 0, 8, fake, fake, fake, None) == 1
    assert lib.moe_route(fake, 4, 4096, 2, 0, 0, 8, fake, fake, fake, None) == 2
    # dispatch: bf16 rows must be multiples of 16 bytes; workspace required for planning
    assert lib.moe_dispatch(fake, 1, 4, 12, 2, fake, None, 0, 4, fake, fake, fake, 0, fake, 8, fake, 1 << 20, None) == 2
    assert lib.moe_dispatch(fake, 1, 4, 16, 2, fake, None, 0, 4, fake, fake, fake, 0, fake, 8, None, 0, None) == 3
    assert lib.moe_dispatch(fake, 5, 4, 16, 2, fake, None, 0, 4, fake, fake, fake, 0, fake, 8, fake, 1 << 20, None) == 1
    # experts: bf16 needs d, f multiples of 64; workspace size is checked
    assert lib.moe_expert_fwd(fake, 1, 8, 96, 64, 2, fake, fake, fake, fake, None, None, None, fake, fake, 1 << 20, None) == 2
    assert lib.moe_expert_fwd(fake, 1, 8, 64, 64, 2, fake, fake, fake, fake, None, None, None, fake, fake, 16, None) == 3
    assert lib.moe_expert_fwd(fake, 1, 8, 64, 64, 2, fake, fake, fake, fake, fake, None, None, fake, fake, 1 << 20, None) == 1
    assert lib.moe_expert_bwd(fake, fake, fake, None, fake, 1, 8, 64, 64, 2, fake, fake, fake, fake, fake, fake, fake, fake,
                              2, fake, 1 << 20, None) == 1
    # a NULL tensor with T > 0 is rejected on the host (it would be dereferenced on the device)
    assert lib.moe_combine(None, 1, 4, 16, 2, fake, None, fake, None) == 1
    assert lib.moe_combine(fake, 1, 4, 16, 2, None, None, fake, None) == 1
    assert lib.moe_combine(fake, 1, 4, 16, 2, fake, None, None, None) == 1
    assert lib.moe_combine_bwd(fake, None, 1, 4, 16, 2, fake, fake, fake, fake, None) == 1
    assert lib.moe_combine_bwd(fake, fake, 1, 4, 16, 2, fake, fake, None, fake, None) == 1
    assert lib.moe_combine_bwd(None, fake, 1, 4, 16, 2, fake, fake, fake, fake, None) == 1
    # fp32 experts: row tiles beyond the grid's second dimension are refused by validation, not by the launch
    assert lib.moe_expert_fwd(fake, 0, 64 * 65536, 64, 64, 2, fake, fake, fake, fake, None, None, None, fake, fake, 1 << 40, None) == 2
    assert lib.moe_combine(fake, 1, 4, 12, 2, fake, None, fake, None) == 2
    # the entry point without a workspace argument refuses plans larger than its built-in scratch:
    # 2^22 tokens x top-8 over 1024 local experts need a 268 MB chunk table
    assert lib.moe_dispatch_static(fake, 1, 1 << 22, 64, 8, fake, None, 0, 1024, fake, fake, fake, fake, 1 << 25, None, None) == 3
    assert B.moe_workspace_bytes(B.WS_DISPATCH, B.MOE_BF16, 1 << 22, 8, 64, 64, 1024, 0) > (4 << 20)
    assert lib.moe_dispatch_static(fake, 1, 4, 12, 2, fake, None, 0, 4, fake, fake, fake, fake, 8, None, None) == 2
    assert lib.moe_dispatch_static(fake, 1, 4, 16, 2, None, None, 0, 4, fake, fake, fake, fake, 8, None, None) == 1
    assert lib.moe_combine(fake, 1, 4, 16, 100, fake, None, fake, None) == 2
