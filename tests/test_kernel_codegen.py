"""Properties of the compiled fused-step kernel that its bandwidth depends on, read from the
assembly hipcc emits for the library's own source (no GPU needed):

  * no scratch memory and at most 256 vector registers (two wavefronts per SIMD must fit);
  * the norm result is read with one scalar load: nothing enters the vector memory pipeline before a
    wavefront's streaming loads (a vector load issued under a saturated stream queues behind it), and
    the result's fields are not fetched one dependent round trip at a time;
  * a full tile issues its eight non-temporal loads back to back, before the first wait on any of them;
  * every streaming access of the full-tile path is non-temporal.
"""
import os
import re
import shutil
import subprocess

import pytest

from paper_2104_07857_amd import build as zb

KERNEL = re.compile(r"^(_ZN2zi17adamw_wide_kernelILi([01])ELb([01])ELb([01])EEEvNS_8StepArgsE):", re.M)


@pytest.fixture(scope="module")
def step_kernels(tmp_path_factory):
    if shutil.which(zb.hipcc()) is None and not os.path.exists(zb.hipcc()):
        pytest.skip("no hipcc here")
    out = tmp_path_factory.mktemp("isa") / "zi_kernels.s"
    flags = [f for f in zb.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [zb.hipcc(), *flags, "-I", os.path.join(zb.ROOT, "include"), "-I", zb.CSRC, "-S", "--cuda-device-only",
           "-o", str(out), os.path.join(zb.CSRC, "zi_kernels.hip")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    text = out.read_text()
    kernels = {}
    for mt in KERNEL.finditer(text):
        end = text.index(".end_amdhsa_kernel", mt.end())
        kernels[(int(mt.group(2)), int(mt.group(3)), int(mt.group(4)))] = text[mt.end():end]
    assert len(kernels) == 8, sorted(kernels)      # {bf16, fp16} x {AdamW, Adam+L2} x {one tensor, list}
    return kernels


def instructions(body):
    out = []
    for line in body.splitlines():
        line = line.split(";")[0].strip()
        if line and not line.startswith(".") and not line.endswith(":"):
            out.append(line)
    return out


def directive(body, name):
    m = re.search(r"\.amdhsa_" + name + r"\s+(\d+)", body)
    assert m, name
    return int(m.group(1))


def test_no_scratch_and_two_wavefronts_per_simd_fit(step_kernels):
    for key, body in step_kernels.items():
        assert directive(body, "private_segment_fixed_size") == 0, key
        assert directive(body, "next_free_vgpr") <= 256, key
        assert "scratch_" not in body and "buffer_" not in body, key


def test_norm_result_is_read_with_one_scalar_load(step_kernels):
    """Up to the prologue's fp64 arithmetic (the clip factor) the kernel has touched memory only through
    scalar loads: its arguments (base s[0:1]) and one 32-byte load of the whole norm result from another
    base; no vector memory instruction, and no field-by-field reads of the result."""
    for key, body in step_kernels.items():
        ins = instructions(body)
        first_f64 = next(i for i, x in enumerate(ins) if x.startswith(("v_div_scale_f64", "v_sqrt_f64", "v_rsq_f64",
                                                                       "v_mul_f64", "v_add_f64")))
        head = ins[:first_f64]
        assert not [x for x in head if x.startswith(("global_", "flat_", "buffer_", "scratch_"))], key
        other = [x for x in head if x.startswith("s_load") and not re.search(r", s\[0:1\], ", x)]
        # (a launch over a list also reads its tensor's descriptor through a computed base, before the result)
        assert (len(other) == 1 or not key[2]) and other, (key, other)
        assert re.match(r"s_load_dwordx8 s\[\d+:\d+\], s\[\d+:\d+\], 0x0$", other[-1]), (key, other)


def test_full_tile_issues_all_loads_before_the_first_wait(step_kernels):
    for key, body in step_kernels.items():
        ins = instructions(body)
        # the full-tile block is the only place with non-temporal 16-byte loads at an immediate offset of one
        # wavefront row (the second quad of a lane)
        start = next(i for i, x in enumerate(ins) if x.startswith("global_load_dwordx") and x.endswith(" nt"))
        loads = 0
        for x in ins[start:]:
            if x.startswith("s_waitcnt") and "vmcnt" in x:
                break
            assert not x.startswith("global_store"), key
            if x.startswith("global_load_dwordx"):
                assert x.endswith(" nt"), (key, x)
                loads += 1
        assert loads == 8, (key, loads)          # 2 quads x (p, m, v, g)
        stores = [x for x in ins[start:] if x.startswith(("global_store_dwordx4", "global_store_dwordx2"))]
        assert len(stores) >= 8 and all(x.endswith(" nt") for x in stores), key
