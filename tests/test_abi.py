"""The C-ABI library loads and exports every symbol the header declares (CPU only:
no device call is made)."""
import ctypes
import os
import re

from paper_2511_09261_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "gco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gco_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(build.LIB):
        build.build(verbose=False)
    lib = ctypes.CDLL(build.LIB)
    names = declared_symbols()
    assert len(names) >= 20
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.exported_symbols()) == names      # the binding mirrors the header


def test_default_config_and_argument_checks_need_no_device():
    lib = binding.load()
    cfg = binding.Config()
    assert lib.gco_default_config(ctypes.byref(cfg)) == binding.OK
    assert (cfg.problem, cfg.num_layers, cfg.dim, cfg.norm, cfg.storage) == (0, 2, 16, 0, 0)
    assert abs(cfg.alpha - 2.0) < 1e-7 and abs(cfg.beta - 1.0) < 1e-7 and abs(cfg.lr - 1e-2) < 1e-9
    assert lib.gco_default_config(None) == binding.EINVAL
    h = ctypes.c_void_p()
    cfg.dim = 24                                            # rejected before any device call
    assert lib.gco_create(ctypes.byref(cfg), ctypes.byref(h)) == binding.EINVAL
    assert lib.gco_num_kernel_kinds() >= 8
    assert lib.gco_kernel_kind_name(0) == b"fwd_hidden"
