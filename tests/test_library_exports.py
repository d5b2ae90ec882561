"""The C-ABI library builds, loads and exports every function include/lgn.h declares.
No compute call is made here (no GPU needed)."""
import ctypes
import os
import re

import paper_2006_08173_amd as lgn
from paper_2006_08173_amd import build as lgn_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "lgn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(lgn_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_header_declares_the_six_path_calls():
    names = _declared_functions()
    for n in ("lgn_stats", "lgn_threshold", "lgn_fp_params", "lgn_prune", "lgn_fp_quantize",
              "lgn_prune_quantize_fused"):
        assert n in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(lgn_build.LIB):
        lgn_build.build(force=True)
    lib = ctypes.CDLL(lgn_build.LIB)
    for name in _declared_functions():
        assert hasattr(lib, name), name
    assert set(_declared_functions()) == set(lgn.EXPORTS)


def test_host_only_helpers():
    assert lgn.lgn_version() == 100
    assert lgn.lgn_packed_bytes(0, 6) == 0
    assert lgn.lgn_packed_bytes(3, 6) == 3
    assert lgn.lgn_packed_bytes(5, 5) == 4
    assert lgn.lgn_packed_bytes(1_000_000_000, 6) == 750_000_000
    assert lgn.lgn_workspace_bytes(10 ** 9, lgn.LGN_BF16) >= 40 * 2048
    # struct layouts match the header's stated sizes
    assert ctypes.sizeof(lgn.LgnStats) == 72
    assert ctypes.sizeof(lgn.LgnPruneParams) == 24
    assert ctypes.sizeof(lgn.LgnFpParams) == 32


def test_tuning_knobs_are_host_state_only():
    for knob, default in ((lgn.LGN_TUNE_STATS_KEEP_MB, 224), (lgn.LGN_TUNE_STATS_BLOCKS_PER_CU, 0),
                          (lgn.LGN_TUNE_STREAM_PAIRS_PER_WAVE, 0), (lgn.LGN_TUNE_STREAM_BLOCKS_PER_CU, 1024),
                          (lgn.LGN_TUNE_STATS_STRICT_PUBLISH, 0)):
        assert lgn.lgn_get_tuning(knob) == default
    lgn.lgn_set_tuning(lgn.LGN_TUNE_STREAM_PAIRS_PER_WAVE, 12)
    assert lgn.lgn_get_tuning(lgn.LGN_TUNE_STREAM_PAIRS_PER_WAVE) == 12
    lgn.lgn_set_tuning(lgn.LGN_TUNE_STREAM_PAIRS_PER_WAVE, -1)
    assert lgn.lgn_get_tuning(lgn.LGN_TUNE_STREAM_PAIRS_PER_WAVE) == 0
    for knob, bad in ((lgn.LGN_TUNE_STATS_KEEP_MB, 5000), (lgn.LGN_TUNE_STREAM_PAIRS_PER_WAVE, 5000),
                      (lgn.LGN_TUNE_STATS_STRICT_PUBLISH, 2), (9, 1)):
        try:
            lgn.lgn_set_tuning(knob, bad)
        except lgn.LgnError as e:
            assert e.code == lgn.LGN_ERR_INVALID_ARG
        else:
            raise AssertionError("accepted a bad knob/value")
    assert lgn.lgn_get_tuning(9) == -1


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2006_08173_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src, os.path.join(dirpath, f)


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asked for more it says so and exits before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
    assert not r.stdout.strip().startswith("{")           # no result line
