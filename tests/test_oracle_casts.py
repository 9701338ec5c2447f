"""Pins for the oracle's casts (round to nearest even, subnormals kept)."""
import os
import subprocess
import tempfile

import numpy as np
import torch

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exhaustive_all_fp32_inputs_against_hardware_and_neighbour_rule():
    """All 2^32 inputs: fp16 vs the CPU's F16C converter, bf16 vs compare-neighbours in double."""
    exe = os.path.join(tempfile.mkdtemp(prefix="zi_cast_"), "cast_exhaustive")
    subprocess.run(["gcc", "-O2", "-fopenmp", "-mf16c", "-mfma", "-ffp-contract=off", "-o", exe,
                    os.path.join(ROOT, "tests", "c", "cast_exhaustive.c"),
                    os.path.join(ROOT, "oracle", "zi_oracle.c"), "-lm"], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "mismatches_f16=0 mismatches_bf16=0" in r.stdout


def _interesting_f32():
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 2**32, size=1_000_000, dtype=np.uint64).astype(np.uint32)
    edges = np.array([0x00000000, 0x80000000, 0x00000001, 0x007FFFFF, 0x00800000, 0x33000000, 0x33000001,
                      0x33800000, 0x387FC000, 0x387FE000, 0x38800000, 0x477FE000, 0x477FEFFF, 0x477FF000,
                      0x477FF001, 0x7F7FFFFF, 0x7F7F8000, 0x7F7F7FFF, 0x7F800000, 0xFF800000,
                      0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001, 0x3F801000, 0x3F803000], dtype=np.uint32)
    return np.concatenate([bits, edges]).view(np.float32)


def test_fp16_matches_numpy_on_a_million_patterns():
    x = _interesting_f32()
    x = x[~np.isnan(x)]
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = oracle.cast(x, oracle.FP16)
    assert np.array_equal(got, want)


def test_bf16_matches_torch_on_a_million_patterns():
    x = _interesting_f32()
    x = x[~np.isnan(x)]
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.cast(x, oracle.BF16)
    assert np.array_equal(got, want)


def test_widen_is_exact_for_every_16_bit_pattern():
    allbits = np.arange(65536, dtype=np.uint16)
    got16 = oracle.widen(allbits, oracle.FP16)
    want16 = allbits.view(np.float16).astype(np.float32)
    assert np.array_equal(got16.view(np.uint32)[~np.isnan(want16)], want16.view(np.uint32)[~np.isnan(want16)])
    assert np.isnan(got16[np.isnan(want16)]).all()
    gotbf = oracle.widen(allbits, oracle.BF16)
    wantbf = torch.from_numpy(allbits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    ok = ~np.isnan(wantbf)
    assert np.array_equal(gotbf.view(np.uint32)[ok], wantbf.view(np.uint32)[ok])
    assert np.isnan(gotbf[~ok]).all()


def test_round_trip_and_monotone_and_ties():
    allbits = np.arange(65536, dtype=np.uint16)
    for dt, nanmask in ((oracle.FP16, lambda b: ((b & 0x7C00) == 0x7C00) & ((b & 0x3FF) != 0)),
                        (oracle.BF16, lambda b: ((b & 0x7F80) == 0x7F80) & ((b & 0x7F) != 0))):
        keep = ~nanmask(allbits)
        back = oracle.cast(oracle.widen(allbits, dt), dt)
        assert np.array_equal(back[keep], allbits[keep])          # idempotent on representables
        assert nanmask(back[~keep]).all()                         # NaN stays NaN
        x = np.sort(np.random.default_rng(3).normal(0, 1, 200000).astype(np.float32))
        y = oracle.widen(oracle.cast(x, dt), dt)
        assert (np.diff(y) >= 0).all()                            # monotone
    # exact ties go to the even neighbour: 1 + 2^-8 lies between bf16 1.0 (even) and 1.0078125 (odd)
    assert oracle.cast(np.array([1.00390625], np.float32), oracle.BF16)[0] == 0x3F80
    assert oracle.cast(np.array([1.01171875], np.float32), oracle.BF16)[0] == 0x3F82
    # fp16: 1 + 2^-11 is a tie between 1.0 (even) and 1+2^-10 (odd); 1 + 3*2^-11 ties up to 1+2^-9
    assert oracle.cast(np.array([1.00048828125], np.float32), oracle.FP16)[0] == 0x3C00
    assert oracle.cast(np.array([1.00146484375], np.float32), oracle.FP16)[0] == 0x3C02
    # overflow: largest finite fp16 is 65504; 65520 is the tie and goes to inf
    assert oracle.cast(np.array([65519.996], np.float32), oracle.FP16)[0] == 0x7BFF
    assert oracle.cast(np.array([65520.0], np.float32), oracle.FP16)[0] == 0x7C00
    # subnormal fp16: 2^-24 is the smallest; 2^-25 ties to zero; just above goes to 2^-24
    assert oracle.cast(np.array([2.0 ** -24], np.float32), oracle.FP16)[0] == 0x0001
    assert oracle.cast(np.array([2.0 ** -25], np.float32), oracle.FP16)[0] == 0x0000
    assert oracle.cast(np.array([np.float32(2.0 ** -25) * np.float32(1.0000001)], np.float32), oracle.FP16)[0] == 0x0001
