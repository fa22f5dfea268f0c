"""Pins for the oracle's number formats: E2M1 node set (paper Sec. 3.1), FP8 E4M3 and bf16
rounding against independent library casts."""
import os

import numpy as np
import torch

from oracle import faar_oracle as fo


def _golden_nodes(golden_dir):
    with open(os.path.join(golden_dir, "e2m1_nodes.txt")) as f:
        return [float(l) for l in f if l.strip() and not l.startswith("#")]


def test_e2m1_codes_enumerate_the_papers_node_set(golden_dir):
    nodes = _golden_nodes(golden_dir)
    vals = fo.e2m1_decode(np.arange(16))
    assert list(vals[:8]) == nodes                       # index-ordered, ascending
    assert list(-vals[8:]) == nodes                      # sign bit mirrors them
    assert np.signbit(vals[8])                           # code 8 is negative zero
    assert list(np.diff(vals[:8])) == [0.5, 0.5, 0.5, 0.5, 1.0, 1.0, 2.0]
    assert list(fo.NODES) == nodes


def test_format_constants(golden_dir):
    kv = {}
    with open(os.path.join(golden_dir, "nvfp4_format.txt")) as f:
        for l in f:
            if l.strip() and not l.startswith("#"):
                k, v = l.split()
                kv[k] = v
    assert fo.BLOCK == int(kv["block_elements"])


def test_e4m3_decode_matches_library_cast_on_every_code():
    b = torch.arange(256, dtype=torch.uint8)
    lib = b.view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    mine = fo.e4m3_decode(b.numpy())
    assert np.array_equal(np.isnan(lib), np.isnan(mine))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], mine[ok])
    assert np.array_equal(np.signbit(lib[ok]), np.signbit(mine[ok]))
    assert fo.E4M3_MAX == 448.0 and fo.E4M3_POS.size == 127
    assert fo.E4M3_POS[1] == 2.0 ** -9 and fo.E4M3_POS[8] == 2.0 ** -6


def test_e4m3_encode_roundtrip_and_saturation():
    assert np.array_equal(fo.e4m3_encode(fo.E4M3_POS.astype(np.float32)), np.arange(127))
    assert fo.e4m3_encode(np.float32(448.0)) == 0x7E
    assert fo.e4m3_encode(np.float32(1e9)) == 0x7E
    assert fo.e4m3_encode(np.float32(464.0)) == 0x7E
    assert fo.e4m3_encode(np.float32(0.0)) == 0
    # hand-checked midpoints: ties go to the even byte
    assert fo.e4m3_encode(np.float32(2.0 ** -10)) == 0          # between 0 and 2^-9
    assert fo.e4m3_encode(np.float32(3 * 2.0 ** -10)) == 2      # between 2^-9 (1) and 2^-8 (2)
    assert fo.e4m3_encode(np.float32(1.0625)) == 0x38           # between 1.0 (0x38) and 1.125 (0x39)
    assert fo.e4m3_encode(np.float32(1.1875)) == 0x3A           # between 1.125 (0x39) and 1.25 (0x3A)
    assert fo.e4m3_encode(np.float32(1.9375)) == 0x40           # between 1.875 (0x3F) and 2.0 (0x40)
    assert fo.e4m3_encode(np.nextafter(np.float32(1.0625), np.float32(2))) == 0x39


def test_e4m3_encode_matches_library_cast():
    rng = np.random.default_rng(5)
    t = np.concatenate([
        rng.uniform(0, 448, 200000), 2.0 ** rng.uniform(-14, 9, 200000),
        rng.uniform(0, 2.0 ** -5, 100000),
        0.5 * (fo.E4M3_POS[:-1] + fo.E4M3_POS[1:]),                # every exact tie
    ]).astype(np.float32)
    t = t[t <= 448.0]                                             # the library cast does not saturate
    lib = torch.from_numpy(t).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(fo.e4m3_encode(t), lib)


def test_bf16_round_matches_library_cast():
    rng = np.random.default_rng(6)
    x = np.concatenate([rng.standard_normal(200000) * 10.0 ** rng.uniform(-30, 30, 200000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -1e-45]]).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    mine = fo.bf16_round(x)
    assert np.array_equal(mine.view(np.uint32), lib.view(np.uint32))
