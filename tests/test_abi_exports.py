"""The C-ABI library loads and exports every symbol include/*.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(x(?:attn|tensor|beam)_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_boundary():
    names = _declared_functions()
    for must in ("xattn_decode", "xtensor_map", "xtensor_unmap", "xattn_last_error", "xbeam_select"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2510_14686_amd import binding
    lib = binding.load_library()
    for name in _declared_functions():
        assert hasattr(lib, name), "libxattn.so does not export %s" % name
    assert sorted(binding.EXPORTS) == _declared_functions()


def test_argument_checks_need_no_gpu():
    """Calls rejected before any GPU work: they only run host code."""
    from paper_2510_14686_amd import binding
    with pytest.raises(binding.XattnError) as e:
        binding.xattn_decode(0, 0, 0, 0, 1, 1, 8, 2, 128, 0.1, 0)
    assert e.value.status == binding.XATTN_EINVAL
    for args, status in (((1, 1, 8, 3, 128), binding.XATTN_EUNSUPPORTED),      # heads not divisible
                         ((1, 1, 8, 2, 64), binding.XATTN_EUNSUPPORTED),       # head_dim
                         ((0, 1, 8, 2, 128), binding.XATTN_EINVAL),            # batch
                         ((1, 17, 8, 2, 128), binding.XATTN_EUNSUPPORTED),     # q_len
                         ((1, 16, 40, 8, 128), binding.XATTN_EUNSUPPORTED)):   # 5 * 16 rows > 64
        with pytest.raises(binding.XattnError) as e:
            binding.xattn_decode(16, 16, 16, 16, *args, 0.1, 16)
        assert e.value.status == status, (args, str(e.value))
        assert binding.xattn_last_error()
    with pytest.raises(binding.XattnError):
        binding.xattn_configure(99, 1)
    with pytest.raises(binding.XattnError):
        binding.xattn_configure(binding.XATTN_CFG_PIECES, -1)
    with pytest.raises(binding.XattnError) as e:
        binding.xtensor_unmap(0)
    assert e.value.status == binding.XATTN_EINVAL


def test_test_hooks_are_not_part_of_the_product_library():
    from paper_2510_14686_amd import binding
    lib = binding.load_library()
    for name in ("xtensor_test_fake_driver", "xtensor_test_fail_next", "xtensor_test_fake_counts", "xattn_test_plan"):
        assert not hasattr(lib, name), name
    assert not any("test" in n for n in _declared_functions())


def test_workspace_sizes_of_both_operators():
    """xattn_workspace_bytes / xattn_mla_workspace_bytes (host arithmetic only): the layouts the header
    states, for the automatic piece count of a device-less process (256) and for a configured one."""
    from paper_2510_14686_amd import binding

    def up(x):
        return (x + 255) // 256 * 256

    binding.xattn_configure(binding.XATTN_CFG_PIECES, 0)
    try:
        for pieces in (0, 40):
            binding.xattn_configure(binding.XATTN_CFG_PIECES, pieces)
            P = pieces or 256
            B, T, Hq = 64, 2, 32
            slots, rows = P + B, T * Hq
            assert binding.xattn_workspace_bytes(B, T, Hq, 8, 128) == up(B * 8) + up(slots * rows * 8) + up(slots * rows * 512)
            # latent-KV: one workgroup per 128 query rows of a sequence works on a piece, and the automatic
            # count gives one workgroup per compute unit
            H = 128
            for Tm in (1, 2, 3):
                rows = Tm * H
                slots = (pieces or 256 // Tm // 8 * 8) + B
                assert binding.xattn_mla_workspace_bytes(B, Tm, H, 512, 64) == up(B * 8) + up(slots * rows * 16) + up(slots * rows * 1024)
    finally:
        binding.xattn_configure(binding.XATTN_CFG_PIECES, 0)
    for bad in ((0, 1, 128, 512, 64), (1, 1, 128, 256, 64), (1, 16, 512, 512, 64), (5000, 1, 8, 512, 64)):
        with pytest.raises(binding.XattnError):
            binding.xattn_mla_workspace_bytes(*bad)
    with pytest.raises(binding.XattnError):
        binding.xattn_workspace_bytes(1, 1, 8, 3, 128)
