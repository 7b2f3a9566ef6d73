"""The C-ABI library loads, exports every symbol include/slp.h declares, and turns
bad arguments into error codes on the host before touching a device.  CPU only."""

import ctypes
import os
import re

import pytest

from paper_2403_11204_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "slp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(slp_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared()
    assert len(names) >= 18
    L = api.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(api.EXPORTS) == names


def _create(widths, act=api.RELU_ALL, loss=api.MSE_SIL, dtype=api.F32, max_batch=8, lr=0.01, mom=0.9):
    L = api.lib()
    arr = (ctypes.c_int * len(widths))(*widths)
    opts = api._Opts(dtype, max_batch, lr, mom, 0)
    h = ctypes.c_void_p()
    rc = L.slp_segment_create(arr, len(widths), act, loss, ctypes.byref(opts), ctypes.byref(h))
    return rc, h


def test_create_rejects_bad_arguments():
    L = api.lib()
    assert _create([4])[0] == -1                       # no layer
    assert _create([4, 0, 3])[0] == -1                 # width <= 0
    assert _create([4, 3], act=7)[0] == -1
    assert _create([4, 3], loss=-2)[0] == -1
    assert _create([4, 3], dtype=5)[0] == -1
    assert _create([4, 3], max_batch=0)[0] == -1
    assert _create([4, 3], mom=1.5)[0] == -1
    assert b"momentum" in L.slp_last_error()
    opts = api._Opts(0, 8, 0.01, 0.9, 0)
    h = ctypes.c_void_p()
    assert L.slp_segment_create(None, 2, 0, 0, ctypes.byref(opts), ctypes.byref(h)) == -1
    # 2^20 x 2^20 weights cannot be addressed
    assert _create([1 << 20, 1 << 20])[0] == -2
    # the limit itself: a weight matrix (its float32 master copy) must stay below 2 GiB (32-bit byte offsets)
    assert _create([23176, 23176], dtype=api.BF16)[0] == -2
    assert b"2 GiB" in L.slp_last_error()
    for dt in (api.F32, api.BF16):
        rc, h = _create([23168, 23168], dtype=dt)                     # 2,147,024,896 bytes: just below
        assert rc == 0
        L.slp_segment_destroy(h)
    assert _create([16, 16], max_batch=(1 << 24) + 1)[0] == -1        # max_batch itself is capped at 2^24
    assert _create([64, 64], max_batch=1 << 24)[0] == -2              # an activation matrix of 4 GiB


def test_sizes_and_state_errors_without_device():
    L = api.lib()
    rc, h = _create([784, 80, 60], max_batch=1410)
    assert rc == 0 and h.value
    pb, wb = L.slp_segment_param_bytes(h), L.slp_segment_workspace_bytes(h)
    # at least master + momentum + gradient for every parameter of the paper's left partition (Sec. 3)
    assert pb >= 3 * 4 * 67660 and pb % 256 == 0
    assert wb >= 4 * 1410 * (784 + 80 + 60) and wb % 256 == 0
    dummy = ctypes.c_void_p(0x1000)
    # nothing bound yet
    assert L.slp_segment_step(h, dummy, dummy, 8, None, None) == -5
    assert L.slp_segment_forward(h, dummy, 8, dummy, None) == -5
    assert L.slp_segment_init(h, 1, None) == -5
    assert L.slp_segment_get_params(h, 0, dummy, dummy, 1, None) == -5
    assert b"bind" in L.slp_last_error()
    # bind validation happens before any device call
    assert L.slp_segment_bind(h, None, pb, dummy, wb, None) == -1
    assert L.slp_segment_bind(h, ctypes.c_void_p(0x1001), pb, ctypes.c_void_p(0x1000), wb, None) == -3
    assert L.slp_segment_bind(h, ctypes.c_void_p(0x1000), pb - 1, ctypes.c_void_p(0x1000), wb, None) == -3
    # labels: wrong width, and a classification segment takes none
    assert L.slp_segment_set_labels(h, dummy, 47, 61) == -2
    assert L.slp_segment_set_labels(h, dummy, 47, 60) == 0
    assert L.slp_segment_set_lr(h, -1.0, 0.9) == -1
    assert L.slp_segment_set_lr(h, 0.1, 0.0) == 0
    L.slp_segment_destroy(h)
    rc, h2 = _create([60, 60, 60, 47], act=api.RELU_HIDDEN_IDENTITY_LAST, loss=api.SOFTMAX_XENT)
    assert rc == 0
    assert L.slp_segment_set_labels(h2, dummy, 47, 47) == -5
    L.slp_segment_destroy(h2)
    assert L.slp_segment_step(None, dummy, dummy, 8, None, None) == -1
    assert L.slp_segment_input_grad(None, dummy, dummy, 8, dummy, None, None) == -1
    assert L.slp_segment_step_external(None, dummy, dummy, 8, None) == -1
    assert L.slp_segment_param_bytes(None) == 0


def test_free_functions_reject_bad_arguments():
    L = api.lib()
    dummy = ctypes.c_void_p(0x1000)
    assert L.slp_make_synthetic_labels(1, 0, 8, 0, 1.0, dummy, 0, None) == -1
    assert L.slp_make_synthetic_labels(1, 4, 8, 9, 1.0, dummy, 0, None) == -1
    assert L.slp_make_synthetic_labels(1, 4, 8, 0, 1.0, None, 0, None) == -1
    assert L.slp_make_synthetic_labels(1, 4, 8, 0, 1.0, dummy, 3, None) == -1
    assert L.slp_make_segment_inputs(1, None, 4, dummy, 0, 2, 8, 0.05, dummy, 0, None) == -1
    assert L.slp_make_segment_inputs(1, dummy, 4, dummy, -1, 2, 8, 0.05, dummy, 0, None) == -1
    tf = ctypes.c_double()
    assert L.slp_probe_mfma_rate(7, 10, dummy, 1 << 22, ctypes.byref(tf), None, None) == -1
    assert L.slp_probe_mfma_rate(1, 0, dummy, 1 << 22, ctypes.byref(tf), None, None) == -1
    assert L.slp_probe_mfma_rate(1, 10, None, 1 << 22, ctypes.byref(tf), None, None) == -1
    assert L.slp_probe_mfma_rate(1, 10, dummy, 1 << 22, None, None, None) == -1


def test_inference_and_switch_calls_reject_bad_arguments():
    L = api.lib()
    dummy = ctypes.c_void_p(0x1000)
    # accuracy count: null pointers, sizes, dtype, scratch too small or misaligned -- all before any launch
    assert L.slp_count_correct(None, dummy, 8, 4, 0, dummy, 64, 0, dummy, None) == -1
    assert L.slp_count_correct(dummy, dummy, 0, 4, 0, dummy, 64, 0, dummy, None) == -1
    assert L.slp_count_correct(dummy, dummy, 8, 4, 9, dummy, 64, 0, dummy, None) == -1
    assert L.slp_count_correct(dummy, dummy, 9, 4, 0, dummy, 8, 0, dummy, None) == -3          # 3 partial counts need 12 bytes
    assert L.slp_count_correct(dummy, dummy, 8, 4, 0, ctypes.c_void_p(0x1002), 64, 0, dummy, None) == -3
    # the allocation-free variant: same argument checks, and its row limit
    assert L.slp_count_correct_static(dummy, None, 8, 4, 0, 0, dummy, None) == -1
    assert L.slp_count_correct_static(dummy, dummy, 8, -1, 0, 0, dummy, None) == -1
    assert L.slp_count_correct_static(dummy, dummy, 65537, 4, 1, 0, dummy, None) == -2
    assert b"65536" in L.slp_last_error()
    assert L.slp_mean_loss(None, 4, dummy, None) == -1
    assert L.slp_mean_loss(dummy, 0, dummy, None) == -1
    # switches on a handle
    assert L.slp_segment_set_fused_update(None, 1) == -1
    rc, h = _create([8, 4])
    assert rc == 0
    assert L.slp_segment_set_fused_update(h, -3) == -1
    assert L.slp_segment_set_fused_update(h, 2) == 0
    n = ctypes.c_int64()
    assert L.slp_segment_target_errors(h, ctypes.byref(n), None) == -5                           # not bound
    assert L.slp_segment_target_errors(None, ctypes.byref(n), None) == -1
    L.slp_segment_destroy(h)


def test_header_is_plain_c(tmp_path):
    # the boundary is C: the header must compile as C99 on its own, and a C caller must link against the library
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_slp.c"
    src.write_text(
        '#include "slp.h"\n'
        '#include <stdio.h>\n'
        'int main(void) {\n'
        '  int widths[3] = {784, 80, 60};\n'
        '  slp_opts o = {SLP_F32, 1410, 0.01f, 0.9f, 0};\n'
        '  slp_segment* seg = NULL;\n'
        '  int rc = slp_segment_create(widths, 3, SLP_RELU_ALL, SLP_MSE_SIL, &o, &seg);\n'
        '  if (rc != SLP_OK) { printf("create failed: %s\\n", slp_last_error()); return 1; }\n'
        '  printf("%zu %zu\\n", slp_segment_param_bytes(seg), slp_segment_workspace_bytes(seg));\n'
        '  rc = slp_segment_step(seg, NULL, NULL, 8, NULL, NULL);   /* not bound, null X: an error code, no crash */\n'
        '  slp_segment_destroy(seg);\n'
        '  return rc < 0 ? 0 : 2;\n'
        '}\n')
    exe = tmp_path / "use_slp"
    libdir = os.path.join(ROOT, "paper_2403_11204_amd")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src),
                    "-o", str(exe), "-L", libdir, "-l:libslp.so", "-Wl,-rpath," + libdir,
                    "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    api_bytes = api.lib().slp_segment_param_bytes  # the same sizes through ctypes
    rc, h = _create([784, 80, 60], max_batch=1410)
    assert rc == 0 and int(out[0]) == api_bytes(h) and int(out[1]) == api.lib().slp_segment_workspace_bytes(h)
    api.lib().slp_segment_destroy(h)
