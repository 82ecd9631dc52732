"""Host-only checks of the C ABI: the library loads without a GPU, exports every
symbol include/monta.h declares, and turns bad arguments into error codes before
any HIP call (so these run on a machine with no GPU)."""
import ctypes
import os
import re

import pytest

import paper_2411_00662_amd as m
from paper_2411_00662_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def good():
    return m.make_cfg(8192, 4096, m.BF16, 8, 2, 8, 1, 4, 2.0)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "monta.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(monta_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations found in the header"
    assert declared == set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_sizes_match_the_header_layout():
    # int64 + 7 * int32 + float + 2 * int32 = 48 bytes; layout: 3 * int64 + 4 * int32 + 16 * int64
    assert ctypes.sizeof(B.monta_cfg) == 48
    assert ctypes.sizeof(B.monta_ws_layout) == 3 * 8 + 4 * 4 + 16 * 8


def test_workspace_query_named_workloads():
    ws, rows = m.monta_workspace_bytes(good())
    assert rows == 16384 and ws > 2 * 8192 * 2 * 4
    L = m.monta_ws_layout_query(m.make_cfg(65536, 7168, m.BF16, 64, 8, 8, 4, 8, 1.25))
    assert L.max_rows == 524288 and L.capacity == 10240 and L.units == 32 and L.tokens_per_unit == 2048
    L = m.monta_ws_layout_query(m.make_cfg(256, 128, m.FP32, 4, 2, 2, 2, 2, 0.0))
    assert L.max_rows == 512 and L.capacity == 256
    L = m.monta_ws_layout_query(m.make_cfg(8192, 4096, m.BF16, 8, 2, 8, 1, 4, 2.0, padded=1))
    assert L.max_rows == 8 * 4096           # padded: E*C rows even though only T*k = 16384 pairs exist
    # cf binds the row bound: E*C < T*k
    L = m.monta_ws_layout_query(m.make_cfg(1024, 64, m.BF16, 4, 2, 2, 1, 1, 0.5))
    assert L.capacity == 256 and L.max_rows == 1024
    offs = [getattr(L, f) for f, _ in B.monta_ws_layout._fields_ if f.startswith("off_")]
    assert offs == sorted(offs) and len(set(offs)) == len(offs) and all(o % 256 == 0 for o in offs)
    assert L.ws_bytes > offs[-1]


@pytest.mark.parametrize("field,value,code", [
    ("tokens", 0, -1), ("hidden", 0, -1), ("experts", 0, -1), ("top_k", 0, -1), ("ep", 0, -1), ("tp", 0, -1),
    ("slices", 0, -1), ("dtype", 2, -1), ("renorm", 2, -1), ("padded", 2, -1), ("padded", -1, -1),
    ("top_k", 9, -1),            # k > E
    ("ep", 3, -1),               # E % ep != 0
    ("slices", 3, -1),           # T % (S*tp) != 0
    ("hidden", 4100, -1),        # row bytes not a multiple of 16 (bf16: 8200)
    ("capacity_factor", -1.0, -1), ("capacity_factor", float("nan"), -1), ("capacity_factor", float("inf"), -1),
])
def test_invalid_cfg_is_rejected(field, value, code):
    cfg = good()
    setattr(cfg, field, value)
    with pytest.raises(m.MontaError) as ei:
        m.monta_workspace_bytes(cfg)
    assert ei.value.code == code


def test_unsupported_limits():
    with pytest.raises(m.MontaError) as ei:
        m.monta_workspace_bytes(m.make_cfg(1024, 64, m.BF16, 512, 2, 1, 1, 1, 0.0))
    assert ei.value.code == -2
    with pytest.raises(m.MontaError) as ei:
        m.monta_workspace_bytes(m.make_cfg(1024, 64, m.BF16, 64, 33, 1, 1, 1, 0.0))
    assert ei.value.code == -2
    with pytest.raises(m.MontaError) as ei:
        m.monta_workspace_bytes(m.make_cfg(2 ** 30, 64, m.BF16, 8, 4, 1, 1, 1, 0.0))   # T*k >= 2^31
    assert ei.value.code == -2


def test_null_and_misaligned_pointers_fail_before_any_gpu_work():
    lib = B.lib()
    cfg = good()
    c = ctypes.byref(cfg)
    fake = 0x1000    # never dereferenced: validation fails first
    assert lib.monta_route(c, 0, fake, fake, fake, 0) == -3
    assert lib.monta_route(c, fake, fake, fake, 0, 0) == -3
    assert lib.monta_route(c, fake + 2, fake, fake, fake, 0) == -5
    assert lib.monta_dispatch(c, 0, fake, fake, 0, 0) == -3
    assert lib.monta_dispatch(c, fake, fake + 8, fake, 0, 0) == -5
    assert lib.monta_dispatch(c, fake, fake, fake, 4, 0) == -1        # slice out of range
    assert lib.monta_dispatch(c, fake, fake, fake, -2, 0) == -1
    assert lib.monta_regather(c, fake, fake, fake, 0, 0) == -1        # in place is not allowed
    assert lib.monta_regather(c, fake, 0, fake, 0, 0) == -3
    assert lib.monta_regather(c, fake, 2 * fake, fake, 7, 0) == -1
    assert lib.monta_dispatch_regather(c, fake, 2 * fake, 0, fake, 0) == -3
    assert lib.monta_dispatch_regather(c, fake, 2 * fake, 2 * fake, fake, 0) == -1
    assert lib.monta_route_dispatch_regather(c, fake, fake, fake, fake, 2 * fake, 3 * fake, 0, 0) == -3
    assert lib.monta_route_dispatch_regather(c, fake, fake, fake, fake, 2 * fake, 2 * fake, fake, 0) == -1
    assert lib.monta_route_dispatch_regather(c, fake, 0, fake, fake, 2 * fake, 3 * fake, fake, 0) == -3
    assert lib.monta_combine(c, fake, 0, 2 * fake, fake, 0) == -3
    assert lib.monta_combine(c, fake, fake, fake, fake, 0) == -1
    assert lib.monta_combine(c, fake, fake, 2 * fake + 4, fake, 0) == -5
    assert lib.monta_allgather(c, fake, fake, fake, 0, 0) == -1
    assert lib.monta_allgather(c, fake, 2 * fake, 0, 0, 0) == -3
    assert lib.monta_allgather(c, fake, 2 * fake, fake, 4, 0) == -1
    assert lib.monta_unregather(c, fake, fake, fake, 0, 0) == -1
    assert lib.monta_unregather(c, fake, 2 * fake, fake, 9, 0) == -1
    assert lib.monta_unregather(c, 0, 2 * fake, fake, 0, 0) == -3
    assert lib.monta_combine_staged(c, fake, 0, 2 * fake, fake, 0, 0) == -3
    assert lib.monta_combine_staged(c, fake, fake, 2 * fake, fake, 4, 0) == -1
    assert lib.monta_combine_staged(c, fake, fake, fake, fake, 0, 0) == -1
    assert lib.monta_unregather_combine(c, fake, fake, fake, 3 * fake, fake, 0) == -1
    assert lib.monta_unregather_combine(c, fake, 2 * fake, fake, 3 * fake, 0, 0) == -3
    assert lib.monta_unregather_combine(c, fake, 2 * fake + 8, fake, 3 * fake, fake, 0) == -5
    assert lib.monta_gate(c, fake, 0, fake, 0) == -3
    assert lib.monta_gate(c, fake, fake, 0, 0) == -3
    assert lib.monta_gate(c, fake + 8, fake, fake, 0) == -5
    assert lib.monta_gate(c, fake, fake, fake + 2, 0) == -5
    assert lib.monta_expert_linear(c, fake, 2 * fake, 4096, 0, fake, -1, 0) == -3
    assert lib.monta_expert_linear(c, fake, 2 * fake, 4096, 3 * fake, fake, 4, 0) == -1
    assert lib.monta_expert_linear(c, fake, 2 * fake, 4100, 3 * fake, fake, 0, 0) == -1      # row of y not whole vectors
    assert lib.monta_expert_linear(c, fake, 2 * fake, 4096, fake, fake, 0, 0) == -1          # in place
    assert lib.monta_expert_linear(c, fake + 4, 2 * fake, 4096, 3 * fake, fake, 0, 0) == -5
    assert lib.monta_route_dispatch_expert(c, fake, fake, fake, fake, 2 * fake, 3 * fake, 4 * fake, 4096, 5 * fake, fake, 2, 0) == -1
    assert lib.monta_route_dispatch_expert(c, fake, fake, fake, fake, 2 * fake, 3 * fake, 0, 4096, 5 * fake, fake, 1, 0) == -3
    assert lib.monta_route_dispatch_expert(c, fake, fake, fake, fake, 2 * fake, 3 * fake, 4 * fake, 4096, 2 * fake, fake, 1, 0) == -1
    assert lib.monta_ws_init(c, 0, 0) == -3
    assert lib.monta_copy(0, fake, 16, 0) == -3
    assert lib.monta_copy(fake, 2 * fake, 24, 0) == -1
    assert lib.monta_copy(fake, 2 * fake + 4, 32, 0) == -5
    assert lib.monta_workspace_bytes(None, None, None) == -3
    assert lib.monta_ws_layout_query(c, None) == -3
    assert lib.monta_profile_read(99, ctypes.byref(ctypes.c_double()), ctypes.byref(ctypes.c_int64())) == -1
    bad = good()
    bad.top_k = 0
    assert lib.monta_route(ctypes.byref(bad), fake, fake, fake, fake, 0) == -1
    assert lib.monta_gate(ctypes.byref(bad), fake, fake, fake, 0) == -1


def test_pipeline_mode_and_strerror():
    assert m.monta_get_pipeline_mode() == -1        # default: chosen per call from the slice size
    old = m.monta_get_pipeline_mode()
    for mode in (-1, 0, 1, 2):
        m.monta_set_pipeline_mode(mode)
        assert m.monta_get_pipeline_mode() == mode
    for bad_mode in (3, -2):
        with pytest.raises(m.MontaError):
            m.monta_set_pipeline_mode(bad_mode)
    m.monta_set_pipeline_mode(old)
    for code in (0, -1, -2, -3, -4, -5, -77):
        assert isinstance(m.monta_strerror(code), str) and m.monta_strerror(code)
    assert m.monta_last_hip_error() == 0


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2411_00662_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2411_00662_amd" not in text and "libmonta.so" not in text


def test_build_refuses_kernels_that_spill():
    """The build reads the compiler's resource-usage remarks and names every kernel that uses scratch memory."""
    from paper_2411_00662_amd.build import scratch_users
    remarks = (
        "k.hpp:1:0: remark: Function Name: kernel_a [-Rpass-analysis=kernel-resource-usage]\n"
        "k.hpp:1:0: remark:     VGPRs: 256 [-Rpass-analysis=kernel-resource-usage]\n"
        "k.hpp:1:0: remark:     ScratchSize [bytes/lane]: 352 [-Rpass-analysis=kernel-resource-usage]\n"
        "k.hpp:9:0: remark: Function Name: kernel_b [-Rpass-analysis=kernel-resource-usage]\n"
        "k.hpp:9:0: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n")
    assert scratch_users(remarks) == [("kernel_a", 352)]
    assert scratch_users("") == []


def test_static_scratch_entry_point_refuses_oversized_problems_on_the_host():
    """The plan tables of 4M pairs do not fit the 16 MiB static array: refused before any GPU call."""
    lib = m.binding.lib()
    cfg = m.make_cfg(1 << 19, 64, m.BF16, 64, 8, 8, 4, 8, 0.0)
    assert m.monta_ws_layout_query(cfg).ws_bytes > (16 << 20)
    fake = ctypes.c_void_p(0x1000)
    rc = lib.monta_route_dispatch_combine_static(ctypes.byref(cfg), fake, fake, fake, fake, ctypes.c_void_p(0x2000),
                                                 ctypes.c_void_p(0x3000), ctypes.c_void_p(0x4000), None)
    assert rc == -6 and "static" in m.monta_strerror(rc)
    # argument checks come first
    assert lib.monta_route_dispatch_combine_static(ctypes.byref(cfg), None, fake, fake, fake, fake, fake, fake, None) == -3


def test_pipeline_query_reports_the_launch_grouping():
    """Host-only: small problems run in three launches (first slice with the plan, the rest as one group),
    slices of 256 MiB and more run one by one as two kernels each, an explicit mode keeps one slice per launch."""
    import workloads
    def q(name, **kw):
        w = workloads.CONFIGS[name].with_(**kw)
        return m.monta_pipeline_query(m.make_cfg(w.tokens, w.hidden, w.dtype, w.experts, w.top_k, w.ep, w.tp, w.slices,
                                                 w.capacity_factor, w.renorm, w.padded))
    assert m.monta_get_pipeline_mode() == -1
    assert q("mixtral") == (1, 1, 3, True)
    assert q("2x70b") == (1, 1, 3, True)
    assert q("longctx") == (2, 1, 1, True)
    assert q("longctx", slices=8) == (2, 2, 2, True)
    assert q("skewed") == (2, 1, 1, False)
    for mode in (0, 1, 2):
        m.monta_set_pipeline_mode(mode)
        assert q("mixtral") == (mode, 1, 1, mode == 1)
    m.monta_set_pipeline_mode(-1)
