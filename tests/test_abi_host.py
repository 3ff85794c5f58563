"""Host-only checks of the boundary (not gpu): the library loads, exports every symbol the header
declares, and its two host functions agree with exact arithmetic.  No kernel is launched."""
import ctypes
import os
import re
from fractions import Fraction
from math import ceil

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "serveflow.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2402_03694_amd import binding, build
    if build.is_stale():
        build.build()
    return binding.load_library()


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sf_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2402_03694_amd import binding
    names = _declared()
    assert {"sf_featurize", "sf_fast_infer", "sf_route", "sf_slow_infer"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_struct_layouts_match_header(tmp_path):
    """The ctypes mirrors must have the layout gcc gives the header's structs."""
    import subprocess
    from paper_2402_03694_amd import binding as b
    fields = {"sf_packets": (b.SfPackets, ["n_flows", "n_pkts", "flow_off", "pkt_size", "pkt_iat", "pkt_dir",
                                           "pkt_hdr", "hdr_words"]),
              "sf_feat_cfg": (b.SfFeatCfg, ["n_windows", "depth", "raw_pkts", "raw_bits"]),
              "sf_forest": (b.SfForest, ["n_trees", "depth", "n_classes", "n_features", "node_feat", "node_thr",
                                         "leaf_label", "packed"]),
              "sf_tree": (b.SfTree, ["depth", "n_classes", "n_features", "node_feat", "node_thr", "leaf_count"]),
              "sf_gbdt": (b.SfGbdt, ["n_trees", "depth", "n_classes", "n_features", "node_feat", "node_thr",
                                     "leaf_value", "base", "packed"]),
              "sf_join_table": (b.SfJoinTable, ["slots", "cap_log2"]),
              "sf_mlp": (b.SfMlp, ["n_in", "n_h1", "n_h2", "n_classes", "dtype", "mu", "inv_sigma", "clamp",
                                   "w1", "w2", "w3", "b1", "b2", "b3", "ordered"])}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "serveflow.h"', 'int main(void){']
    for name, (_, fs) in fields.items():
        lines.append('printf("%s %%zu\\n", sizeof(%s));' % (name, name))
        for f in fs:
            lines.append('printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (name, f, name, f))
    lines.append("return 0;}")
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    got = dict(l.split() for l in subprocess.check_output([str(exe)], text=True).splitlines())
    for name, (cls, fs) in fields.items():
        assert ctypes.sizeof(cls) == int(got[name]), name
        for f in fs:
            assert getattr(cls, f).offset == int(got["%s.%s" % (name, f)]), (name, f)


def test_vmin_from_theta_exact(lib):
    for theta in (0.0, 0.1, 0.25, 0.3, 1 / 3, 0.5, 0.7, 0.75, 0.9, 1.0):
        for T in (1, 7, 16, 100, 200, 500, 65535):
            want = min(65535, ceil(Fraction(float(np.float32(theta))) * T))
            assert lib.sf_vmin_from_theta(ctypes.c_float(theta), T) == want, (theta, T)
    assert lib.sf_vmin_from_theta(ctypes.c_float(-1.0), 10) == 0
    assert lib.sf_vmin_from_theta(ctypes.c_float(2.0), 65535) == 65535


def test_workspace_bytes_monotone(lib):
    a = lib.sf_workspace_bytes(4096, 16, 8, 32, 128, 128)
    b = lib.sf_workspace_bytes(1 << 20, 100, 12, 64, 512, 512)
    c = lib.sf_workspace_bytes(1 << 20, 100, 12, 0, 0, 0)
    d = lib.sf_workspace_bytes(1 << 20, 100, 12, 4800, 1024, 512)
    assert d - lib.sf_workspace_bytes(1 << 20, 100, 12, 64, 1024, 512) >= (4800 - 64) * 1024 * 2   # ordered first-layer weights
    assert 0 < a < b and c < b and a % 256 == 0 and b % 256 == 0
    assert c >= 100 * 1365 * 16         # the packed forest alone: (4^6-1)/3 two-level records of 16 bytes per tree


def test_create_rejects_bad_arguments_without_gpu(lib):
    h = ctypes.c_void_p()
    assert lib.sf_create(None, None, None, 0) == -1
    assert lib.sf_create(ctypes.byref(h), None, None, 1 << 20) == -1
    assert b"workspace" in lib.sf_last_error(None)
    assert lib.sf_create(ctypes.byref(h), None, ctypes.c_void_p(0x1001), 1 << 20) == -1
    assert b"aligned" in lib.sf_last_error(None)
    # entry points refuse a NULL context instead of crashing
    assert lib.sf_featurize(None, None, None, None, 0, None) == -1
    assert lib.sf_fast_infer(None, None, 0, 0, None, None, None, None, None) == -1
    assert lib.sf_route(None, None, None, 0, None, 0, None, None) == -1
    assert lib.sf_slow_infer(None, None, 0, None, None, None, None, 0, 0, None, None, None, None) == -1


def test_product_package_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2402_03694_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "libsf_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2402_03694_amd" not in text and "serveflow.h" not in text, f
