"""The GPU entry points called from C: a strict-C99 translation unit that includes only include/zi.h,
built with the box's C compiler into a shared object, loaded into this process and handed the device
buffers as plain addresses.  The arrays it leaves behind are compared with the oracle."""
import ctypes
import os
import shutil
import subprocess

import numpy as np
import pytest
import torch

import oracle
import paper_2104_07857_amd as zi
import zi_synth
from gpu_util import NormBuffers, TOL_NORM_REL, compare_state, gen_numpy, progress, to_dev, to_np

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


class ClientArgs(ctypes.Structure):
    _fields_ = [("p", ctypes.c_uint64), ("m", ctypes.c_uint64), ("v", ctypes.c_uint64), ("g", ctypes.c_uint64),
                ("p_lp", ctypes.c_uint64), ("numel", ctypes.c_int64), ("d_norm", ctypes.c_uint64),
                ("d_norm2", ctypes.c_uint64), ("d_workspace", ctypes.c_uint64), ("workspace_bytes", ctypes.c_uint64),
                ("hip_stream", ctypes.c_uint64), ("lp_dtype", ctypes.c_int32), ("step", ctypes.c_int32),
                ("loss_scale", ctypes.c_float), ("max_grad_norm", ctypes.c_float)]


@pytest.fixture(scope="module")
def client(tmp_path_factory):
    cc = shutil.which("gcc") or shutil.which("cc") or shutil.which("clang")
    if cc is None:
        pytest.skip("no C compiler on this box (looked for gcc, cc, clang)")
    so = str(tmp_path_factory.mktemp("cclient") / "libzi_c_client.so")
    libdir = os.path.dirname(zi.LIB_PATH)
    subprocess.run([cc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-O1", "-fPIC", "-shared",
                    "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c", "abi_gpu_client.c"),
                    "-o", so, "-L", libdir, "-lzi", "-Wl,-rpath," + libdir], check=True)
    zi.lib()                                     # the library itself is already in the process
    L = ctypes.CDLL(so)
    L.zi_c_client_run.restype = ctypes.c_int
    L.zi_c_client_run.argtypes = [ctypes.POINTER(ClientArgs), ctypes.c_char_p, ctypes.c_size_t]
    return L


@pytest.mark.parametrize("dt,loss_scale", [(zi.ZI_BF16, 1.0), (zi.ZI_FP16, 1024.0)])
def test_resident_path_called_from_c(client, dt, loss_scale):
    n = 70_003
    spec = zi_synth.StateSpec(31337 + dt, dt, g_std=1e-3 * loss_scale)
    hp, hm, hv, hg = gen_numpy(spec, n)
    p, m, v, g = to_dev(hp), to_dev(hm), to_dev(hv), to_dev(hg)
    lp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    nb, nb2 = NormBuffers(), NormBuffers()
    args = ClientArgs(p.data_ptr(), m.data_ptr(), v.data_ptr(), g.data_ptr(), lp.data_ptr(), n,
                      nb.out.data_ptr(), nb2.out.data_ptr(), nb.ws.data_ptr(), nb.ws.numel(),
                      torch.cuda.current_stream().cuda_stream, dt, 10, loss_scale, 0.05)
    err = ctypes.create_string_buffer(512)
    rc = client.zi_c_client_run(ctypes.byref(args), err, 512)
    torch.cuda.synchronize()
    assert rc == 0, f"C client: code {rc}: {err.value.decode()}"
    sumsq, flag = oracle.grad_sumsq([hg], dt)
    cfg = oracle.config(step=10, loss_scale=loss_scale, max_grad_norm=0.05)
    lpe = np.zeros(n, np.uint16)
    oracle.adamw(hp, hm, hv, hg, lpe, dt, cfg, sumsq, flag)
    for got in (nb.read(), nb2.read()):
        assert got[2] == flag == 0
        want = np.sqrt(sumsq) / loss_scale
        assert abs(got[1] - want) <= TOL_NORM_REL * want
    assert nb.read()[0] == nb2.read()[0]
    progress("C client: " + compare_state((hp, hm, hv, lpe), (to_np(p), to_np(m), to_np(v), to_np(lp)), dt))
