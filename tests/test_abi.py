"""Host-only checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import pytest

from paper_2212_05231_amd import binding as nb
from paper_2212_05231_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "neus2.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(neus2_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 15
    handle = C.CDLL(nb.LIB_PATH)
    for name in names:
        assert hasattr(handle, name), name
    assert set(names) == set(nb.EXPORTS)
    assert nb.lib().neus2_version() >= 1


def test_struct_layout_matches_header():
    # 5 ints + 2*32 ints + (1+5) + (1+5) ints + 2 ints + 2 floats
    assert C.sizeof(nb.Neus2Config) == 4 * (5 + 64 + 6 + 6 + 2 + 4)
    assert C.sizeof(nb.Neus2StepBuffers) == 8 * 34


def test_struct_sizes_against_the_c_compiler(tmp_path):
    """sizeof of the header's structs as gcc sees them equals the ctypes mirrors'."""
    import subprocess
    src = tmp_path / "sizes.c"
    src.write_text('#include <stdio.h>\n#include "neus2.h"\n'
                   'int main(void) { printf("%zu %zu\\n", sizeof(neus2_config), sizeof(neus2_step_buffers)); return 0; }\n')
    exe = tmp_path / "sizes"
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run(["gcc", "-I", inc, str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(v) for v in out] == [C.sizeof(nb.Neus2Config), C.sizeof(nb.Neus2StepBuffers)]


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_benchmark_descriptors_validate(k):
    assert nb.validate_config(nb.make_config(wl.make_config(k))) == 0


def test_bad_descriptors_are_rejected_with_a_message():
    def broken(**kw):
        cfg = wl.make_config(2)
        c = nb.make_config(cfg)
        for name, v in kw.items():
            setattr(c, name, v)
        return c
    cases = [
        (broken(n_levels=0), -3), (broken(n_levels=33), -3), (broken(n_features=4), -5),
        (broken(log2_table_size=30), -3), (broken(active_levels=17), -3), (broken(table_dtype=2), -3),
        (broken(n_sdf_mats=5), -5), (broken(samples_per_ray=65), -3), (broken(loss_kind=3), -3), (broken(loss_kind=2, huber_delta=0.0), -3),
        (broken(s=0.0), -3), (broken(frozen_levels=17), -3), (broken(beta=-1.0), -3),
    ]
    c = broken()
    c.dense[15] = 1          # (2049)^3 vertices do not fit 2^19 slots
    cases.append((c, -3))
    c = broken()
    c.sdf_dims[1] = 128
    cases.append((c, -5))
    for c, code in cases:
        assert nb.validate_config(c) == code
        assert len(nb.lib().neus2_last_error()) > 0
    assert nb.lib().neus2_validate_config(None) == -1


def test_null_and_misaligned_pointers_are_rejected_before_any_launch():
    L = nb.lib()
    c = nb.make_config(wl.make_config(2))
    ok = 0x1000
    assert L.neus2_hash_encode(C.byref(c), None, ok, 10, ok, ok, None, None) == -1
    assert b"pos" in L.neus2_last_error()
    assert L.neus2_hash_encode(C.byref(c), ok, ok, 10, ok + 4, ok, None, None) == -4
    assert L.neus2_hash_encode(C.byref(c), ok, ok, -1, ok, ok, None, None) == -2
    assert L.neus2_sdf_fwd_grad(C.byref(c), ok, ok, None, 10, ok, ok, ok, None, None) == -1
    assert L.neus2_color_fwd(C.byref(c), ok, ok, ok, None, ok, None, 64, ok, None, None) == -1
    arr = (C.c_void_p * 3)(ok, ok, ok)
    assert L.neus2_color_fwd(C.byref(c), ok, ok, ok, None, ok, arr, 63, ok, None, None) == -2     # not a multiple of 64
    assert L.neus2_color_fwd(C.byref(c), ok, ok, ok, None, ok, arr, 64, ok, ok + 2, None) == -4    # masks misaligned
    assert L.neus2_render_rays(C.byref(c), ok, 0, ok, None, 4, ok, ok, None) == -2
    assert L.neus2_loss(C.byref(c), ok, ok, ok, ok, 3, 100, ok, ok, ok, ok, None) == -2
    assert L.neus2_adam_step(ok, None, ok, ok, ok, 10, 1, 0.01, 0.9, 0.99, 1e-15, 1, 1, None) == -1   # fp16 needs master
    assert L.neus2_adam_step(ok, None, ok, ok, ok, 10, 0, 0.01, 0.9, 0.99, 1e-15, 0, 1, None) == -3   # t starts at 1
    # flag bit 2 (leave out the levels beyond the active ones) belongs to the table calls only
    assert L.neus2_adam_step(ok, None, ok, ok, ok, 10, 0, 0.01, 0.9, 0.99, 1e-15, 1, 4, None) == -3
    assert b"flags" in L.neus2_last_error()
    assert L.neus2_adam_tables(C.byref(c), ok, ok, ok, ok, ok, 0.01, 0.9, 0.99, 1e-15, 1, 8, None) == -3
    assert L.neus2_adam_tables(C.byref(c), ok, None, ok, ok, ok, 0.01, 0.9, 0.99, 1e-15, 1, 4, None) == -1   # fp16 tables need master
    assert L.neus2_rigid_fwd(ok, None, None, 1.0, 0.0, 10, ok, None) == -1
    assert L.neus2_train_step(C.byref(c), None, 64, None) == -1


def _step_buffers(ok, mats):
    b = nb.Neus2StepBuffers()
    for name, _ in nb.Neus2StepBuffers._fields_:
        if name not in ("workspace_bytes", "n_rays", "H", "W", "dH", "dW", "workspace", "s_dev", "d_s", "ray_offsets",
                        "sample_ray", "d_pos", "sdf_masks", "color_masks"):
            setattr(b, name, ok)
    for name in ("H", "W", "dH", "dW"):
        setattr(b, name, C.cast(mats, C.c_void_p))
    return b


def test_train_step_checks_every_buffer_before_its_first_launch():
    """A NULL or misaligned field anywhere in the step's buffers is reported before anything is
    launched: on a host without a GPU the call returns the pointer error, not a launch error."""
    L = nb.lib()
    c = nb.make_config(wl.make_config(2))
    ok = 0x1000
    mats = (C.c_void_p * 3)(ok, ok, ok)
    for field in ("dW", "dH", "W", "H", "d_tables", "rgb", "d_rgb", "dC", "weights", "d_enc", "q", "target", "dirs"):
        b = _step_buffers(ok, mats)
        setattr(b, field, None)
        assert L.neus2_train_step(C.byref(c), C.byref(b), 128, None) == -1, field
        assert field.encode() in L.neus2_last_error()
    broken = (C.c_void_p * 3)(ok, None, ok)
    b = _step_buffers(ok, mats)
    b.dW = C.cast(broken, C.c_void_p)
    assert L.neus2_train_step(C.byref(c), C.byref(b), 128, None) == -1 and b"dW[1]" in L.neus2_last_error()
    b = _step_buffers(ok, mats)
    b.color_masks = ok + 8
    assert L.neus2_train_step(C.byref(c), C.byref(b), 128, None) == -4
    b = _step_buffers(ok, mats)
    assert L.neus2_train_step(C.byref(c), C.byref(b), 100, None) == -2          # not a multiple of 64 samples


def test_workload_generators_are_seeded_and_in_range():
    import numpy as np
    a = wl.make_workload(2, n_rays=16)
    b = wl.make_workload(2, n_rays=16)
    assert np.array_equal(a["batch"]["pos"], b["batch"]["pos"])
    assert np.array_equal(a["params"]["tables"], b["params"]["tables"])
    pos = a["batch"]["pos"]
    assert pos.dtype == np.float32 and pos.min() >= 0 and pos.max() < 1
    assert np.allclose(np.linalg.norm(a["batch"]["dirs"], axis=1), 1, atol=1e-6)
    assert a["params"]["tables"].dtype == np.float16 and abs(a["params"]["tables"]).max() <= 1e-4 + 1e-7
    assert wl.make_config(2).res == [16, 22, 30, 42, 58, 80, 111, 153, 212, 294, 406, 561, 776, 1072, 1482, 2048]
    assert wl.make_config(1).res == [16, 24, 36, 54, 81, 121, 182, 273]
    assert wl.make_config(4).dense[:7] == [1, 1, 1, 1, 1, 1, 0]
