"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the header declares,
its host-side arithmetic (Eq. 6-7 quotas, workspace sizes) is right, and argument errors are reported
before anything reaches a GPU.  No compute call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch  # noqa: F401  (loaded first so that the library binds to the same HIP runtime)

from oracle import metok_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "metok.h")
LIB = os.path.join(ROOT, "paper_2506_02850_amd", "libmetok.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2506_02850_amd import build
        build.build(verbose=False)
    lib = ctypes.CDLL(LIB)
    lib.metok_last_error.restype = ctypes.c_char_p
    return lib


def declared_symbols():
    text = open(HEADER).read()
    return re.findall(r"METOK_API\s+[\w\s\*]+?\b(metok_\w+)\s*\(", text)


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert len(names) == 28 and len(set(names)) == len(names)
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in metok.h but not exported"
    from paper_2506_02850_amd import binding
    assert sorted(binding.EXPORTS) == sorted(names)


def test_header_cites_the_paper_for_every_call():
    text = open(HEADER).read()
    for needle in ("Sec. 3.2.1", "Eq. 4", "Eq. 5", "Algorithm 1", "Sec. 3.2.2", "Eq. 6-7", "Sec. 3.3", "Eq. 3"):
        assert needle in text


def test_retention_quotas_match_eq_6_7(lib):
    f = lib.metok_retention_quotas
    f.argtypes = [ctypes.c_int, ctypes.c_double, ctypes.c_double, ctypes.c_int64, ctypes.c_int64, ctypes.POINTER(ctypes.c_int32)]
    out = (ctypes.c_int32 * 2)()
    rng = np.random.default_rng(0)
    for _ in range(200):
        level = int(rng.integers(0, 4))
        r, alpha = float(rng.uniform(0.05, 1.0)), float(rng.uniform(0.05, 1.0))
        nk, nn = int(rng.integers(0, 40000)), int(rng.integers(0, 40000))
        assert f(level, r, alpha, nk, nn, out) == 0
        assert (out[0], out[1]) == O.retention_quotas(level, r, alpha, nk, nn)
    # the paper's LongVA setting (r = 0.55, alpha = 0.5) by hand
    assert f(1, 0.55, 0.5, 10000, 8432, out) == 0 and (out[0], out[1]) == (5500, 2319)
    assert f(2, 0.55, 0.5, 10000, 8432, out) == 0 and (out[0], out[1]) == (3025, 0)
    assert f(3, 0.55, 0.5, 10000, 8432, out) == 0 and (out[0], out[1]) == (0, 0)
    assert f(4, 0.55, 0.5, 1, 1, out) == -1 and b"level" in lib.metok_last_error()
    assert f(1, 0.0, 0.5, 1, 1, out) == -1
    assert f(1, 0.5, 1.5, 1, 1, out) == -1


def test_account_matches_the_oracle_on_random_settings():
    """metok_account is host arithmetic: it runs without a GPU and must agree with the oracle field by field."""
    from paper_2506_02850_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(5))
    for _ in range(200):
        k = int(rng.integers(1, 14))
        lens = [int(x) for x in rng.integers(1, 30, size=k)]
        keys = [int(x) for x in rng.integers(0, 2, size=k)]
        gh, gw = int(rng.integers(1, 30)), int(rng.integers(1, 30))
        alpha, beta, r = (float(rng.choice([0.25, 0.3, 0.5, 0.55, 0.76, 1.0])) for _ in range(3))
        s1, s2 = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        edge = int(rng.integers(0, 2))
        L = int(rng.integers(1, 41))
        lh = sorted(int(x) for x in rng.integers(0, L + 3, size=3))
        n_text = int(rng.integers(0, 200))
        got = B.metok_account(lens, keys, gh, gw, alpha, beta, s1, s2, edge, r, lh, L, n_text)
        want = O.account(lens, keys, (gh, gw), alpha, beta, s1, s2, edge, r, lh, L, n_text)
        assert got == want, (lens, keys, gh, gw, alpha, beta, s1, s2, edge, r, lh, L, n_text)
    with pytest.raises(B.MetokError):
        B.metok_account([3, 0], [1, 0], 4, 4, 0.5, 0.5, 2, 3, 0, 0.5, [1, 2, 3], 4, 5)        # empty event
    with pytest.raises(B.MetokError):
        B.metok_account([3], [1], 4, 4, 0.5, 0.5, 2, 3, 0, 0.5, [3, 2, 1], 4, 5)              # layers not ascending


def test_workspace_queries(lib):
    seg = lib.metok_segment_events_workspace_bytes
    seg.restype = ctypes.c_size_t
    seg.argtypes = [ctypes.c_int] * 4
    # LongVA-shaped stage 1: 144 wave chunks of four tokens x 3 partials x 4 bytes per frame, two per-frame arrays,
    # and for the pooled reading of Eq. 4 the fp32 frame means with their own (one chunk) partials
    assert seg(256, 576, 1024, 1) == 256 * 144 * 3 * 4 + 2 * 1024 + 256 * 1024 * 4 + 256 * 3 * 4
    assert seg(256, 576, 1020, 1) == 0            # d not a multiple of 8
    assert seg(8, 16, 64, 0) > 0
    prune = lib.metok_prefill_prune_workspace_bytes
    prune.restype = ctypes.c_size_t
    prune.argtypes = [ctypes.c_int64] + [ctypes.c_int] * 6
    full = prune(36992, 28, 4, 128, 64, 36864, 1)
    no_attention = prune(36992, 0, 0, 0, 0, 36864, 1)
    assert full > no_attention > 36864
    assert full < 8 << 20                         # a few MB: partial column sums dominate
    kvw = lib.metok_kv_compact_workspace_bytes
    kvw.restype = ctypes.c_size_t
    kvw.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_int]
    # LongVA-shaped cache: tiles of 512 rows (1024 threads x 8 pieces of a 256-byte row), 73 per slab, 64 slabs per
    # layer, one 4-byte flag each, after a 256-byte header (error word, one ticket per launch)
    assert kvw(28, 8, 4, 36992, 128, 1) == 256 + 28 * 64 * 73 * 4
    assert kvw(28, 8, 4, 36992, 12, 1) == 0       # 24-byte rows


def test_argument_errors_before_any_launch(lib):
    vp, i32, i64, sz, dbl = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t, ctypes.c_double
    seg = lib.metok_segment_events
    seg.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    fake = 0x1000                                   # aligned, never dereferenced: validation fails first
    assert seg(None, 1, 8, 16, 64, None, 2, 0, fake, fake, fake, None, fake, 1 << 20, None) == -1
    assert seg(fake, 1, 8, 16, 64, None, 9, 0, fake, fake, fake, None, fake, 1 << 20, None) == -1       # k > T
    assert b"k must be" in lib.metok_last_error()
    assert seg(fake, 1, 8, 16, 64, None, 2, 7, fake, fake, fake, None, fake, 1 << 20, None) == -1       # sim_mode
    assert seg(fake, 1, 8, 16, 64, None, 2, 0, fake, fake, fake, None, fake, 16, None) == -3            # workspace
    assert seg(fake, 1, 8, 16, 64, None, 2, 0, fake, fake, fake, fake, fake, 1 << 20, None) == -1       # score without text
    assert seg(fake, 3, 8, 16, 64, None, 2, 0, fake, fake, fake, None, fake, 1 << 20, None) == -1       # dtype
    assert seg(fake, 1, 9000, 16, 64, None, 2, 0, fake, fake, fake, None, fake, 1 << 30, None) == -1    # T limit
    kv = lib.metok_kv_compact
    kv.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(vp), i32, i32, i32, i64, i32, i32, ctypes.POINTER(vp),
                   ctypes.POINTER(ctypes.c_int32), vp, vp, sz, vp]
    k = (vp * 1)(fake); v = (vp * 1)(fake); idx = (vp * 1)(fake)
    nk = (ctypes.c_int32 * 1)(4)
    assert kv(k, v, 1, 1, 1, 16, 12, 1, idx, nk, None, fake, 1 << 20, None) == -1      # 24-byte rows
    assert kv(k, v, 1, 1, 1, 16, 16, 1, idx, nk, None, fake, 16, None) == -3           # workspace too small
    assert kv(k, v, 1, 1, 1, 16, 16, 1, idx, nk, None, None, 0, None) == -3            # no workspace
    nk[0] = 17
    assert kv(k, v, 1, 1, 1, 16, 16, 1, idx, nk, None, fake, 1 << 20, None) == -1      # n_keep > S_cap
    assert kv(k, v, 0, 1, 1, 16, 16, 1, idx, nk, None, fake, 1 << 20, None) == -1      # L < 1
    assert kv(k, v, 200, 1, 1, 16, 16, 1, idx, nk, None, fake, 1 << 20, None) == -1    # L > METOK_MAX_LAYERS
    kvp = lib.metok_kv_compact_paged
    kvp.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(vp), i32, i32, i32, i64, i32, i32, i32, vp, i32, ctypes.POINTER(vp),
                    ctypes.POINTER(ctypes.c_int32), vp, vp, sz, vp]
    nk[0] = 4
    assert kvp(k, v, 1, 1, 1, 8, 4, 16, 1, None, 4, idx, nk, None, fake, 1 << 20, None) == -1      # no page table
    assert kvp(k, v, 1, 1, 1, 8, 0, 16, 1, fake, 4, idx, nk, None, fake, 1 << 20, None) == -1      # page_size < 1
    nk[0] = 17
    assert kvp(k, v, 1, 1, 1, 8, 4, 16, 1, fake, 4, idx, nk, None, fake, 1 << 20, None) == -1      # n_keep > pages_per_seq * page_size
    one = lib.metok_segment_compress
    one.argtypes = [vp, i32, i32, i32, i32, i32, vp, i32, i32, dbl, dbl, i32, i32, i32, i32, vp, vp, vp, vp, i64, i32,
                    vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    args = [fake, 1, 8, 4, 4, 64, fake, 2, 0, 1.0, 1.0, 2, 2, 0, 0, fake, fake, fake, fake, 8 * 4, 1] + [fake] * 7 + [fake, 1 << 22, None]
    bad = list(args); bad[6] = None
    assert one(*bad) == -1 and b"text_emb" in lib.metok_last_error()                 # Eq. 5 needs the text embedding
    bad = list(args); bad[7] = 9
    assert one(*bad) == -1 and b"k must be" in lib.metok_last_error()                # k > T on the one-pass path
    bad = list(args); bad[19] = 31
    assert one(*bad) == -4                                                           # out_tokens too small
    bad = list(args); bad[10] = 1.5
    assert one(*bad) == -1                                                           # beta > 1
    bad = list(args); bad[11] = 3; bad[7] = 9
    assert one(*bad) == -1 and b"k must be" in lib.metok_last_error()                # same check on the two-pass path
    bad = list(args); bad[-2] = 16
    assert one(*bad) == -3                                                           # workspace
    copy = lib.metok_calib_copy
    copy.argtypes = [vp, vp, sz, vp]
    assert copy(fake, fake, 24, None) == -1


def test_presets_hold_the_appendix_settings(tmp_path):
    """Appendix "Implementation Details": (s1, s2) = (2, 3) and alpha = 0.5 everywhere; L_H = [3, 10, 19] for the Qwen-based
    models, [13, 24, 34] for VILA; k / beta / r = 5 / 0.4 / 0.76 (LLaVA-OneVision), 13 / 0.45 / 0.55 (LongVA),
    3 / 0.4 / 0.65 (VILA); 24 / 28 / 28 / 40 layers; 32 / 32 / 128 / 16 frames."""
    from paper_2506_02850_amd import binding as B
    from paper_2506_02850_amd import synth
    want = {
        B.MODEL_LLAVA_OV_0_5B: dict(frames=32, n_layers=24, k=5, s1=2, s2=3, layers_h=[3, 10, 19], alpha=0.5, beta=0.4, r=0.76),
        B.MODEL_LLAVA_OV_7B: dict(frames=32, n_layers=28, k=5, s1=2, s2=3, layers_h=[3, 10, 19], alpha=0.5, beta=0.4, r=0.76),
        B.MODEL_LONGVA_7B: dict(frames=128, n_layers=28, k=13, s1=2, s2=3, layers_h=[3, 10, 19], alpha=0.5, beta=0.45, r=0.55),
        B.MODEL_VILA_13B: dict(frames=16, n_layers=40, k=3, s1=2, s2=3, layers_h=[13, 24, 34], alpha=0.5, beta=0.4, r=0.65),
    }
    for model, params in want.items():
        assert B.metok_preset(model) == params
    with pytest.raises(B.MetokError):
        B.metok_preset(4)
    # the shapes the chained model tests run are these presets
    ov, vila = B.metok_preset(B.MODEL_LLAVA_OV_7B), B.metok_preset(B.MODEL_VILA_13B)
    for sh, pr in ((synth.OV_7B, ov), (synth.VILA_13B, vila)):
        assert (sh.n_events, sh.n_layers, list(sh.L_H)) == (pr["k"], pr["n_layers"], pr["layers_h"])
        assert (sh.extra["alpha"], sh.extra["beta"], sh.extra["r"], sh.extra["s1"], sh.extra["s2"]) == (
            pr["alpha"], pr["beta"], pr["r"], pr["s1"], pr["s2"])
    # the header is plain C and the initialiser macros agree with metok_preset(): compile and run a C program
    src = tmp_path / "presets.c"
    src.write_text(
        '#include <stdio.h>\n#include "metok.h"\n'
        "int main(void) {\n"
        "  const metok_params p[4] = {METOK_PRESET_LLAVA_OV_0_5B, METOK_PRESET_LLAVA_OV_7B, METOK_PRESET_LONGVA_7B, METOK_PRESET_VILA_13B};\n"
        "  for (int i = 0; i < 4; ++i) printf(\"%d %d %d %d %d %d %d %d %.2f %.2f %.2f\\n\", p[i].frames, p[i].n_layers, p[i].k, p[i].s1,\n"
        "    p[i].s2, p[i].layers_h[0], p[i].layers_h[1], p[i].layers_h[2], p[i].alpha, p[i].beta, p[i].r);\n"
        "  return 0; }\n")
    exe = tmp_path / "presets"
    import subprocess
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    lines = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.strip().splitlines()
    for model, line in enumerate(lines):
        pr = want[model]
        assert line == "%d %d %d %d %d %d %d %d %.2f %.2f %.2f" % (pr["frames"], pr["n_layers"], pr["k"], pr["s1"], pr["s2"],
                                                                     *pr["layers_h"], pr["alpha"], pr["beta"], pr["r"])


def test_capacity_rows_is_the_worst_case_of_the_pooling_plan():
    from paper_2506_02850_amd import binding as B
    cap = B.metok_compress_encoder_tokens_capacity_rows
    assert cap(32, 24, 24, 2, 3) == 32 * 144                       # every frame a key frame of a key event
    assert cap(32, 27, 27, 2, 3, B.POOL_FLOOR) == 32 * 169 and cap(32, 27, 27, 2, 3, B.POOL_CEIL) == 32 * 196
    assert cap(8, 4, 4, 9, 7) == 8                                  # strides clamp to the grid: one token per frame
    rng = np.random.Generator(np.random.PCG64(11))
    for _ in range(100):
        T, gh, gw = int(rng.integers(1, 50)), int(rng.integers(1, 30)), int(rng.integers(1, 30))
        s1, s2, edge = int(rng.integers(1, 7)), int(rng.integers(1, 7)), int(rng.integers(0, 2))
        # the oracle's row count of a frame pooled with the smaller stride, for every frame
        s = min(max(min(s1, s2), 1), max(gh, gw))
        assert cap(T, gh, gw, s1, s2, edge) == T * O.pooled_side(gh, s, edge) * O.pooled_side(gw, s, edge)
    with pytest.raises(ValueError):
        cap(0, 4, 4, 2, 2)


def test_static_scratch_call_refuses_shapes_beyond_its_array(lib):
    """The entry point without a workspace argument checks the size before it touches the device."""
    from paper_2506_02850_amd import binding as B
    blib = B.lib()
    # 40 kv heads x 200 000 visual keys need 32 MB of column partials alone
    need = blib.metok_prefill_prune_workspace_bytes(200064, 40, 40, 128, 64, 200000, B.BF16)
    assert need > B.metok_static_scratch_bytes() == 8 << 20
    quota = (ctypes.c_int32 * 1)(10)
    fake = 0x1000
    rc = blib.metok_prefill_prune_static(fake, 200064, 8, B.BF16, fake, fake, 40, 40, 128, 64, 0, 0, 200000, fake, fake, None, 0,
                                         1, quota, None, fake, fake, fake, None, None, None, None)
    assert rc == -3 and "static array" in B.metok_last_error()


def test_binding_refuses_cpu_tensors():
    from paper_2506_02850_amd import binding
    with pytest.raises(ValueError):
        binding.metok_segment_events(torch.zeros((4, 4, 64)), 2)
    with pytest.raises(TypeError):
        binding.metok_segment_events(torch.zeros((4, 4, 64), dtype=torch.float16), 2)


def test_product_path_does_not_touch_the_oracle():
    """The oracle is test infrastructure: nothing under the package may import it."""
    pkg = os.path.join(ROOT, "paper_2506_02850_amd")
    pat = re.compile(r"^\s*(from|import)\s+oracle\b|metok_oracle|oracle[/\\.]", re.M)
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, name)).read()
                assert not pat.search(text), f"{name} refers to the oracle"
    # and the oracle does not import the package's binding or library
    text = open(os.path.join(ROOT, "oracle", "metok_oracle.py")).read()
    assert "binding" not in text and "libmetok" not in text and "ctypes" not in text


def test_bench_refuses_more_than_one_gpu():
    """The measurement is one GPU's: bench.py says so and exits instead of timing anything at --gpus 2."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
