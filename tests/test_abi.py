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


def test_workgroup_apportionment_is_exact_within_bounds():
    """Host side of the work decomposition (gco_apportion): the shares add up to the target
    exactly when the bounds allow, respect the bounds, follow the weights, and the answer is
    the hand-computed one on a small case."""
    import numpy as np
    # hand case: weights 5 : 3 : 2 of 7 units -> floors 3, 2, 1 (sum 6), the seventh goes where
    # work per unit is largest: 5/4 = 1.25, 3/3 = 1, 2/2 = 1 -> the first
    got = binding.apportion([5.0, 3.0, 2.0], 7, [0, 0, 0], [9, 9, 9])
    assert got.tolist() == [4, 2, 1]
    # a lower bound of one unit each forces 3 of 4 units onto near-empty parts; the rest follows
    got = binding.apportion([100.0, 0.1, 0.1, 0.1], 6, [1, 1, 1, 1], [50, 50, 50, 50])
    assert got.tolist() == [3, 1, 1, 1]
    # an upper bound caps the heavy part, the remainder goes to the next heaviest per unit
    got = binding.apportion([100.0, 10.0, 10.0], 12, [1, 1, 1], [4, 20, 20])
    assert got.tolist() == [4, 4, 4]
    # outside the feasible range the nearest bound is returned
    assert binding.apportion([1.0, 1.0], 1, [1, 1], [5, 5]).tolist() == [1, 1]
    assert binding.apportion([1.0, 1.0], 99, [1, 1], [5, 5]).tolist() == [5, 5]
    rs = np.random.RandomState(5)
    for target in (512, 1536, 3072):
        work = rs.pareto(1.5, 64) * 1e4 + 50.0              # skewed, like subgraph sizes
        tiles = np.maximum(1, (work / 40).astype(np.int32))
        got = binding.apportion(work, target, np.ones(64, np.int32), tiles)
        assert got.sum() == min(target, tiles.sum())
        assert (got >= 1).all() and (got <= tiles).all()
        free = (got > 1) & (got < tiles)                    # shares no bound touches follow the weights
        per_unit = work[free] / got[free]
        assert per_unit.max() / per_unit.min() < 1.0 + 2.0 / got[free].min()
        assert (binding.apportion(work, target, np.ones(64, np.int32), tiles) == got).all()
    lib = binding.load()
    assert lib.gco_apportion(None, 0, 0, None, None, None) == binding.EINVAL
