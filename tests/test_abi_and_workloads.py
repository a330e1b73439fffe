"""CPU-side checks: the C-ABI library loads and exports what include/z2z.h declares; the binding agrees
with the header's constants; the input generators are deterministic and in range."""
import ctypes
import os
import re

import numpy as np

from paper_2506_01084_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "z2z.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(z2z_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2506_01084_amd import api

    names = _declared_functions()
    assert "z2z_lzw_encode" in names and "z2z_lzw_decode" in names
    assert "z2z_hyper_embed" in names and "z2z_extended_logits" in names
    assert os.path.exists(api.LIB_PATH), "build the library first: python -m paper_2506_01084_amd.build"
    lib = ctypes.CDLL(api.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in z2z.h but not exported"
    assert sorted(api.EXPORTS) == names, "binding and header disagree on the exported calls"
    lib.z2z_strerror.restype = ctypes.c_char_p
    assert lib.z2z_strerror(0) == b"ok" and b"invalid" in lib.z2z_strerror(-1)


def test_binding_constants_match_header():
    from paper_2506_01084_amd import api

    text = open(HEADER).read()

    def enum_value(name):
        m = re.search(r"\b%s\s*=\s*(-?\d+)" % name, text)
        assert m, name
        return int(m.group(1))

    assert api.F32 == enum_value("Z2Z_F32") and api.BF16 == enum_value("Z2Z_BF16")
    assert api.POOL_MEAN == enum_value("Z2Z_POOL_MEAN") and api.POOL_WEIGHTED == enum_value("Z2Z_POOL_WEIGHTED")
    assert api.APPEND == enum_value("Z2Z_APPEND") and api.RESET == enum_value("Z2Z_RESET")
    assert api.ST_BAD_TOKEN == enum_value("Z2Z_ST_BAD_TOKEN") and api.ST_BAD_CODE == enum_value("Z2Z_ST_BAD_CODE")
    assert api.ST_OVERFLOW == enum_value("Z2Z_ST_OVERFLOW")
    for k in ("LOGITS_KERNEL", "LOGITS_STRIP", "LZW_KERNEL", "DECODE_KERNEL", "TIMING", "LOGITS_MAP", "SAMPLE_KERNEL"):
        assert getattr(api, "OPT_" + k) == enum_value("Z2Z_OPT_" + k)
    assert api.MAX_M == int(re.search(r"#define\s+Z2Z_MAX_M\s+(\d+)", text).group(1))
    # the config struct mirrors the header field for field
    fields = [f[0] for f in api.Config._fields_]
    assert fields == ["B", "V", "M", "cap", "d", "dtype", "pool", "w"]
    assert ctypes.sizeof(api.Config) == 7 * 4 + 4 * api.MAX_M
    # the encoder structs: field names and order as in the header
    body = re.search(r"typedef struct z2z_encoder_layer \{(.*?)\} z2z_encoder_layer;", text, re.S).group(1)
    names = re.findall(r"\*\s*(\w+);", body)
    assert names == [f[0] for f in api.EncoderLayer._fields_]
    body = re.search(r"typedef struct z2z_encoder \{(.*?)\} z2z_encoder;", text, re.S).group(1)
    names = re.findall(r"(\w+);", body)
    assert names == [f[0] for f in api.EncoderDesc._fields_]
    assert ctypes.sizeof(api.EncoderLayer) == 12 * ctypes.sizeof(ctypes.c_void_p)
    assert ctypes.sizeof(api.EncoderDesc) == 4 * 4 + 2 * ctypes.sizeof(ctypes.c_void_p)


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 on its own, and the structs have the binding's sizes."""
    import subprocess

    src = tmp_path / "t.c"
    src.write_text('#include "z2z.h"\n#include <stdio.h>\nint main(void) { printf("%zu %zu %zu\\n", sizeof(z2z_config), '
                   'sizeof(z2z_encoder_layer), sizeof(z2z_encoder)); return 0; }\n')
    exe = tmp_path / "t"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.dirname(HEADER), str(src), "-o",
                    str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    from paper_2506_01084_amd import api

    assert [int(x) for x in out] == [ctypes.sizeof(api.Config), ctypes.sizeof(api.EncoderLayer), ctypes.sizeof(api.EncoderDesc)]


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2506_01084_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", src, flags=re.M), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            src = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2506_01084_amd" not in src, f


def test_token_generators_are_seeded_and_in_range():
    for name in ("c1", "c2", "c4", "c5"):
        cfg = wl.scaled(wl.CONFIGS[name], B=2, N=2000)
        a, b = wl.make_tokens(cfg), wl.make_tokens(cfg)
        assert a.dtype == np.int32 and a.shape == (2, 2000)
        assert (a == b).all()
        assert a.min() >= 0 and a.max() < cfg["V"]
        other = wl.make_tokens(wl.scaled(cfg, seed=cfg["seed"] + 100))
        assert (a != other).any()
    lens = wl.make_lens(wl.scaled(wl.CONFIGS["c1"], B=8), ragged=True)
    assert lens[0] == 512 and lens[1] == 0 and lens[2] == 1 and (lens >= 0).all() and (lens <= 512).all()


def test_planted_repeats_compress_inside_the_papers_band():
    """Synthetic streams stand in for real text: their LZW compression rate should sit in the range the
    paper reports for real corpora (13-41 % fewer tokens; merge-size table 68-75 % at M = 2..5), loosely."""
    import oracle

    rates = {}
    for name in ("c1", "c2", "c4", "c5"):
        cfg = wl.scaled(wl.CONFIGS[name], B=1)
        x = wl.make_tokens(cfg)[0].tolist()
        codes, entries, st = oracle.lzw_encode(x, cfg["V"], cfg["M"], cfg["cap"])
        rates[name] = len(codes) / len(x)
    assert 0.80 < rates["c1"] < 0.97
    assert 0.70 < rates["c2"] < 0.90
    assert 0.55 < rates["c4"] < 0.80
    assert 0.50 < rates["c5"] < 0.70


def test_dense_generators_shapes_dtypes_and_thread_independence():
    a = wl.normal_matrix(5, 300, 64, 0.02, "f32", threads=1)
    b = wl.normal_matrix(5, 300, 64, 0.02, "f32", threads=4)
    assert a.dtype == np.float32 and (a == b).all()
    assert abs(float(a.std()) - 0.02) < 0.002
    c = wl.normal_matrix(5, 300, 64, 0.02, "bf16")
    assert c.dtype == np.uint16 and c.shape == (300, 64)
    # bf16 bits are the rounded float32 values: the widened value is within half an ulp (2^-9 relative)
    import oracle
    back = oracle.bf16_bits_to_f64(c)
    assert (np.abs(back - a) <= np.abs(a) * 2.0 ** -8 + 1e-30).all()
    w = wl.make_pool_weights(wl.CONFIGS["c5"])
    assert w.shape == (8,) and (w[5:] == 0).all() and (w[:5] != 0).all()
    assert (wl.make_pool_weights(wl.CONFIGS["c2"]) == 0).all()
    rows = wl.sample_rows(wl.scaled(wl.CONFIGS["c2"], B=3), 100, 5)
    assert len(rows) == 15 and set([0, 99, 100, 199, 200, 299]) <= set(rows.tolist())
    codes = wl.make_step_codes(wl.CONFIGS["c3"], np.array([0, 5, 4096]), 0)
    V = wl.CONFIGS["c3"]["V"]
    assert codes[0] < V and 0 <= codes[1] < V + 5 and 0 <= codes[2] < V + 4096


def test_bench_refuses_more_than_one_gpu():
    """The benchmark is single-GPU: asking for more exits with a message, before anything touches a device."""
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "single-GPU" in (r.stdout + r.stderr)
