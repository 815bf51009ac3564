"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol the header
declares, and rejects bad arguments before any HIP call."""
import ctypes
import os
import re

import pytest

import paper_2601_17917_amd as sd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sd.LIB_PATH):
        from paper_2601_17917_amd.build import build
        build(verbose=False)
    return sd.load_library()


def test_exports_every_declared_symbol(lib):
    import glob
    declared = set()
    for path in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        header = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)
        declared |= set(re.findall(r"\b(sdllm_[a-z0-9_]+)\s*\(", header))
    assert declared == set(sd.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.sdllm_version() == 200
    # the method's header carries no diagnostics
    main = open(os.path.join(ROOT, "include", "sdllm.h")).read()
    assert "sdllm_probe_" not in re.sub(r"/\*.*?\*/", "", main, flags=re.S)


def test_headers_compile_as_plain_c_and_a_c_program_links(tmp_path, lib):
    """The boundary is a C ABI: both headers compile as C99 without warnings, and a plain C program links against
    the library and calls it (host-only entry points: no GPU needed)."""
    import shutil, subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "c.c"
    src.write_text('''#include <stdio.h>
#include "sdllm.h"
#include "sdllm_diag.h"
int main(void) {
  sdllm_attn_params a = {SDLLM_BF16, 4, 32, 32, 128, 5120, 6144, 64, 960, 64, 0.0f, 0};
  sdllm_attn_plan pl;
  int32_t idx[80], n = 0;
  if (sdllm_version() != SDLLM_VERSION) return 1;
  if (sdllm_plan_attention(&a, &pl) != SDLLM_OK || pl.kv_splits != 2 || pl.workgroups != 256) return 2;
  if (sdllm_suffix_keep_indices(960, 64, 1, 1, idx, 80, &n) != SDLLM_OK || n != 65 || idx[63] != 63 || idx[64] != 959) return 3;
  a.D = 96;
  if (sdllm_plan_attention(&a, &pl) != SDLLM_ERR_UNSUPPORTED || sdllm_last_error()[0] == 0) return 4;
  if (sdllm_probe_read(NULL, 0, NULL, NULL) != SDLLM_ERR_INVALID_ARG) return 5;
  printf("ok %s\\n", sdllm_status_string(SDLLM_OK));
  return 0;
}
''')
    exe = tmp_path / "c_prog"
    libdir = os.path.dirname(sd.LIB_PATH)
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                        str(src), "-o", str(exe), "-L", libdir, "-l:libsdllm.so", "-Wl,-rpath," + libdir,
                        "-Wl,-rpath,/opt/rocm/lib"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.startswith("ok ok"), (r.returncode, r.stdout, r.stderr[-500:])


def test_struct_layouts_match_header():
    assert ctypes.sizeof(sd.AttnParams) == 12 * 4
    assert ctypes.sizeof(sd.UnmaskParams) == 48
    assert sd.UnmaskParams.ld.offset == 16
    assert ctypes.sizeof(sd.AppendParams) == 48
    assert sd.AppendParams.cache_layer_stride.offset == 32
    assert ctypes.sizeof(sd.AttnPlan) == 24
    assert ctypes.sizeof(sd.LmHeadPlan) == 28
    assert ctypes.sizeof(sd.LmHeadParams) == 64
    assert sd.LmHeadParams.ld_h.offset == 16 and sd.LmHeadParams.tau0.offset == 32


def test_status_strings(lib):
    assert lib.sdllm_status_string(0) == b"ok"
    assert b"workspace" in lib.sdllm_status_string(sd.ERR_WORKSPACE)


def _attn(lib, p, ptrs=None, ws=(None, 0)):
    vp = ctypes.c_void_p
    ptrs = ptrs or [vp(4096)] * 10
    return lib.sdllm_block_attention(ctypes.byref(p), *ptrs, ws[0], ws[1], None)


@pytest.mark.parametrize("kw,status", [
    (dict(Hq=3, Hkv=2), sd.ERR_INVALID_ARG),
    (dict(prefix_len=100, prefix_cap=64), sd.ERR_INVALID_ARG),
    (dict(n_keep=5, S=4), sd.ERR_INVALID_ARG),
    (dict(D=96), sd.ERR_UNSUPPORTED),
    (dict(dtype=7), sd.ERR_UNSUPPORTED),
    (dict(K=0), sd.ERR_INVALID_ARG),
    (dict(kv_splits=-1), sd.ERR_INVALID_ARG),
])
def test_attention_validation(lib, kw, status):
    base = dict(dtype=sd.BF16, B=1, Hq=4, Hkv=4, D=128, prefix_len=64, prefix_cap=64, K=32, S=32, n_keep=8,
                scale=0.0, kv_splits=0)
    base.update(kw)
    p = sd.attn_params(**base)
    assert _attn(lib, p) == status
    assert lib.sdllm_last_error() != b""
    assert lib.sdllm_attention_workspace_bytes(ctypes.byref(p)) == ctypes.c_size_t(-1).value


def test_attention_null_misaligned_and_workspace(lib):
    vp = ctypes.c_void_p
    p = sd.attn_params(sd.BF16, 1, 4, 4, 128, 640, 640, 32, 32, 8, 0.0, 3)
    ptrs = [vp(4096)] * 10
    bad = list(ptrs); bad[0] = None
    assert _attn(lib, p, bad) == sd.ERR_INVALID_ARG              # q_block NULL
    bad = list(ptrs); bad[2] = None
    assert _attn(lib, p, bad) == sd.ERR_INVALID_ARG              # cache NULL with prefix_len > 0
    bad = list(ptrs); bad[8] = None
    assert _attn(lib, p, bad) == sd.ERR_INVALID_ARG              # keep_idx NULL with n_keep > 0
    bad = list(ptrs); bad[4] = vp(4100)
    assert _attn(lib, p, bad) == sd.ERR_INVALID_ARG              # misaligned
    need = lib.sdllm_attention_workspace_bytes(ctypes.byref(p))
    assert need == 1 * 4 * 40 * 3 * 130 * 4
    assert _attn(lib, p, ptrs, (None, 0)) == sd.ERR_WORKSPACE
    assert _attn(lib, p, ptrs, (vp(8192), need - 1)) == sd.ERR_WORKSPACE
    assert b"workspace" in lib.sdllm_last_error()


def test_plan_is_consistent(lib):
    for (B, Hq, Hkv, P, K, S, s) in [(1, 32, 32, 608, 32, 128, 32), (8, 32, 32, 1024, 32, 992, 32),
                                      (8, 32, 32, 1024, 32, 992, 992), (16, 28, 4, 512, 32, 224, 32),
                                      (4, 32, 32, 5120, 64, 960, 64), (1, 1, 1, 0, 1, 0, 0)]:
        p = sd.attn_params(sd.BF16, B, Hq, Hkv, 128, P, max(P, 1), K, S, s)
        pl = sd.plan_attention(p)
        key_tiles = -(-(P + K + s) // 64)
        assert pl.kv_splits >= 1 and pl.key_tiles_per_split >= 1
        assert (pl.kv_splits - 1) * pl.key_tiles_per_split < key_tiles <= pl.kv_splits * pl.key_tiles_per_split
        rows = (Hq // Hkv) * (K + s)
        q_tiles = -(-rows // pl.rows_per_workgroup)
        assert pl.workgroups >= B * Hkv * pl.kv_splits * q_tiles
        ws = sd.attention_workspace_bytes(p)
        assert ws == (0 if pl.kv_splits == 1 else B * Hq * (K + s) * pl.kv_splits * 130 * 4)


def test_plan_invariants_over_random_parameters(lib):
    """Host-only: for a few hundred seeded random parameter sets the plan covers every key tile exactly once with
    non-empty splits, launches enough workgroups for every (K/V head, split, query tile), uses the 8-wave shapes
    only where they are built for, and the workspace query matches it."""
    import numpy as np
    g = np.random.Generator(np.random.Philox(key=2024))
    seen = set()
    for _ in range(400):
        D = int(g.choice([64, 128])); Hkv = int(g.integers(1, 33)); ratio = int(g.choice([1, 2, 4, 7, 8]))
        B = int(g.integers(1, 17)); K = int(g.choice([1, 16, 32, 64])); P = int(g.integers(0, 9000))
        S = int(g.choice([0, 32, 224, 992])); s = int(g.integers(0, S + 1)); splits = int(g.choice([0, 0, 0, 1, 2, 5]))
        p = sd.attn_params(sd.BF16, B, ratio * Hkv, Hkv, D, P, max(P, 1), K, S, s, 0.0, splits)
        pl = sd.plan_attention(p)
        key_tiles = -(-(P + K + s) // 64)
        rows = ratio * (K + s)
        assert 1 <= pl.kv_splits <= max(key_tiles, 1) and pl.key_tiles_per_split >= 1
        assert (pl.kv_splits - 1) * pl.key_tiles_per_split < key_tiles <= pl.kv_splits * pl.key_tiles_per_split
        if splits:
            assert pl.kv_splits <= splits
        q_tiles = -(-rows // pl.rows_per_workgroup)
        assert pl.workgroups >= B * Hkv * pl.kv_splits * q_tiles and pl.workgroups % 8 == 0
        assert pl.workgroup_shape in (0, 1, 2) and 2 <= pl.ring_stages <= 4
        if pl.workgroup_shape == 2:
            assert rows >= 512 and pl.rows_per_workgroup in (128, 256)
        if pl.workgroup_shape == 1:
            assert pl.workgroups <= 256 and pl.key_tiles_per_split >= 4 and pl.ring_stages == 2
        ws = sd.attention_workspace_bytes(p)
        assert ws == (0 if pl.kv_splits == 1 else B * ratio * Hkv * (K + s) * pl.kv_splits * (D + 2) * 4)
        seen.add(pl.workgroup_shape)
    assert seen == {0, 1, 2}


def test_plan_picks_the_workgroup_shape_from_the_parameters(lib):
    """Host-only: which of the three workgroup shapes a launch takes.  One workgroup per CU at most and splits
    of >= 4 key tiles: two groups on the same rows; K/V heads with >= 512 query rows: two groups on different rows
    sharing the tiles (256 rows per workgroup, three ring stages); everything else: the 4-wave workgroup."""
    def plan(B, Hq, Hkv, P, K, S, s, splits=0):
        return sd.plan_attention(sd.attn_params(sd.BF16, B, Hq, Hkv, 128, P, max(P, 1), K, S, s, 0.0, splits))
    cfg5 = plan(4, 32, 32, 5120, 64, 960, 64)
    assert (cfg5.workgroup_shape, cfg5.kv_splits, cfg5.rows_per_workgroup, cfg5.workgroups) == (1, 2, 128, 256)
    cfg3a = plan(8, 32, 32, 1024, 32, 992, 32)
    assert (cfg3a.workgroup_shape, cfg3a.kv_splits, cfg3a.rows_per_workgroup) == (1, 1, 64)
    cfg3b = plan(8, 32, 32, 1024, 32, 992, 992)
    assert (cfg3b.workgroup_shape, cfg3b.rows_per_workgroup, cfg3b.ring_stages, cfg3b.workgroups) == (2, 256, 3, 1024)
    cfg4 = plan(16, 28, 4, 512, 32, 224, 32)
    assert (cfg4.workgroup_shape, cfg4.rows_per_workgroup, cfg4.ring_stages) == (0, 64, 2)
    cfg2 = plan(1, 32, 32, 608, 32, 128, 32)
    assert cfg2.workgroup_shape == 0 and cfg2.key_tiles_per_split < 4        # three tiles per split: too short to share
    fp32 = sd.plan_attention(sd.attn_params(sd.FP32, 1, 4, 4, 64, 64, 64, 32, 224, 16))
    assert fp32.workgroup_shape == 0


@pytest.mark.parametrize("kw,status", [
    (dict(V=0), sd.ERR_INVALID_ARG),
    (dict(ld=100, V=126464), sd.ERR_INVALID_ARG),
    (dict(ld=126465, V=126464), sd.ERR_INVALID_ARG),       # row stride not a multiple of 16 bytes
    (dict(K=5000), sd.ERR_UNSUPPORTED),
    (dict(dtype=3), sd.ERR_UNSUPPORTED),
    (dict(r_extra_masked=5, r_extra_total=4), sd.ERR_INVALID_ARG),
])
def test_unmask_validation(lib, kw, status):
    base = dict(dtype=sd.BF16, B=2, K=32, V=126464, ld=126464, tau0=0.9, alpha=0.3)
    base.update(kw)
    p = sd.unmask_params(**base)
    vp = ctypes.c_void_p
    rc = lib.sdllm_confidence_unmask(ctypes.byref(p), vp(4096), vp(4096), vp(4096), None, vp(4096), vp(4096), None,
                                     vp(4096), 1 << 30, None)
    assert rc == status


def test_unmask_null_and_workspace(lib):
    vp = ctypes.c_void_p
    p = sd.unmask_params(sd.BF16, 2, 32, 126464, 126464, 0.9, 0.3)
    need = sd.unmask_workspace_bytes(p)
    assert need > 0 and need % 12 == 0
    args = [vp(4096), vp(4096), vp(4096), None, vp(4096), vp(4096), None]
    assert lib.sdllm_confidence_unmask(ctypes.byref(p), *args, vp(4096), need - 1, None) == sd.ERR_WORKSPACE
    assert lib.sdllm_confidence_unmask(ctypes.byref(p), *args, None, need, None) == sd.ERR_WORKSPACE
    bad = list(args); bad[1] = None
    assert lib.sdllm_confidence_unmask(ctypes.byref(p), *bad, vp(4096), need, None) == sd.ERR_INVALID_ARG


@pytest.mark.parametrize("kw,status", [
    (dict(V=0), sd.ERR_INVALID_ARG),
    (dict(Hd=4100), sd.ERR_UNSUPPORTED),                     # not a multiple of 32
    (dict(ld_h=4000), sd.ERR_INVALID_ARG),                   # row stride below the width
    (dict(ld_w=4100), sd.ERR_INVALID_ARG),                   # row stride not a multiple of 16 bytes
    (dict(K=5000), sd.ERR_UNSUPPORTED),
    (dict(B=4096, K=32), sd.ERR_UNSUPPORTED),                # more than 65536 positions
    (dict(r_extra_masked=5, r_extra_total=4), sd.ERR_INVALID_ARG),
    (dict(tau0=float("nan")), sd.ERR_INVALID_ARG),
])
def test_lm_head_validation(lib, kw, status):
    base = dict(B=2, K=32, V=126464, Hd=4096, ld_h=4096, ld_w=4096, tau0=0.9, alpha=0.3)
    base.update(kw)
    p = sd.lm_head_params(**base)
    vp = ctypes.c_void_p
    rc = lib.sdllm_lm_head_unmask(ctypes.byref(p), vp(4096), vp(4096), vp(4096), vp(4096), None, vp(4096), vp(4096),
                                  None, vp(4096), 1 << 30, None)
    assert rc == status
    assert lib.sdllm_last_error() != b""
    assert lib.sdllm_lm_head_unmask_workspace_bytes(ctypes.byref(p)) == ctypes.c_size_t(-1).value


def test_lm_head_null_misaligned_and_workspace(lib):
    vp = ctypes.c_void_p
    p = sd.lm_head_params(1, 32, 126464, 4096, 4096, 4096, 0.9, 0.3)
    need = sd.lm_head_unmask_workspace_bytes(p)
    assert need > 0 and need % (32 * 12) == 0                 # one (max, sum, arg-max) triple per position and vocabulary tile
    args = [vp(4096), vp(4096), vp(4096), vp(4096), None, vp(4096), vp(4096), None]
    assert lib.sdllm_lm_head_unmask(ctypes.byref(p), *args, vp(4096), need - 1, None) == sd.ERR_WORKSPACE
    assert lib.sdllm_lm_head_unmask(ctypes.byref(p), *args, None, need, None) == sd.ERR_WORKSPACE
    for i in (0, 1, 2, 3, 5, 6):
        bad = list(args); bad[i] = None
        assert lib.sdllm_lm_head_unmask(ctypes.byref(p), *bad, vp(4096), need, None) == sd.ERR_INVALID_ARG
    bad = list(args); bad[1] = vp(4104)
    assert lib.sdllm_lm_head_unmask(ctypes.byref(p), *bad, vp(4096), need, None) == sd.ERR_INVALID_ARG
    assert lib.sdllm_lm_head_unmask(None, *args, vp(4096), need, None) == sd.ERR_INVALID_ARG


@pytest.mark.parametrize("kw,status", [
    (dict(prefix_len=40, K=32, prefix_cap=64), sd.ERR_INVALID_ARG),
    (dict(D=4, dtype=sd.BF16), sd.ERR_UNSUPPORTED),           # 8-byte rows
    (dict(n_layers=0), sd.ERR_INVALID_ARG),
    (dict(cache_layer_stride=8), sd.ERR_INVALID_ARG),
])
def test_append_validation(lib, kw, status):
    base = dict(dtype=sd.BF16, n_layers=2, B=1, Hkv=2, D=128, K=32, prefix_len=0, prefix_cap=64,
                cache_layer_stride=0, block_layer_stride=0)
    base.update(kw)
    p = sd.AppendParams(**base)
    vp = ctypes.c_void_p
    assert lib.sdllm_kv_append(ctypes.byref(p), vp(4096), vp(4096), vp(4096), vp(4096), None, None) == status


def test_binding_refuses_host_tensors(lib):
    import torch
    x = torch.zeros((1, 1, 32, 128), dtype=torch.bfloat16)
    with pytest.raises(sd.SdllmError):
        sd.block_attention(x, None, None, None, x, x, None, None, None, 0)


@pytest.mark.parametrize("kw,status", [
    (dict(D=40), sd.ERR_UNSUPPORTED),
    (dict(D=1024), sd.ERR_UNSUPPORTED),
    (dict(dtype=5), sd.ERR_UNSUPPORTED),
    (dict(n_keep=9, S=8), sd.ERR_INVALID_ARG),
    (dict(pos0=-1), sd.ERR_INVALID_ARG),
    (dict(pos0=2**31 - 10), sd.ERR_INVALID_ARG),
    (dict(theta_base=1.0), sd.ERR_INVALID_ARG),
    (dict(theta_base=float("nan")), sd.ERR_INVALID_ARG),
    (dict(K=0), sd.ERR_INVALID_ARG),
])
def test_rope_validation(lib, kw, status):
    base = dict(dtype=sd.BF16, B=1, H=2, D=128, K=32, S=64, n_keep=8, pos0=100, theta_base=10000.0, interleaved=0)
    base.update(kw)
    p = sd.RopeParams(**base)
    vp = ctypes.c_void_p
    assert lib.sdllm_rope_gathered(ctypes.byref(p), vp(4096), vp(4096), vp(4096), vp(4096), vp(4096), None) == status
    assert lib.sdllm_last_error() != b""


def test_rope_null_and_misaligned(lib):
    vp = ctypes.c_void_p
    p = sd.RopeParams(sd.FP32, 1, 2, 64, 4, 8, 2, 0, 10000.0, 0)
    ok = [vp(4096)] * 5
    for i in (0, 1, 2, 3, 4):
        bad = list(ok); bad[i] = None
        assert lib.sdllm_rope_gathered(ctypes.byref(p), *bad, None) == sd.ERR_INVALID_ARG
    bad = list(ok); bad[3] = vp(4100)
    assert lib.sdllm_rope_gathered(ctypes.byref(p), *bad, None) == sd.ERR_INVALID_ARG
    assert lib.sdllm_rope_gathered(None, *ok, None) == sd.ERR_INVALID_ARG
    assert ctypes.sizeof(sd.RopeParams) == 40


def test_validate_keep_idx_host_side(lib):
    vp = ctypes.c_void_p
    assert lib.sdllm_validate_keep_idx(None, 0, 10, None) == sd.SDLLM_OK            # empty list: nothing to read
    assert lib.sdllm_validate_keep_idx(None, 3, 10, None) == sd.ERR_INVALID_ARG
    assert lib.sdllm_validate_keep_idx(vp(4096), 11, 10, None) == sd.ERR_INVALID_ARG  # more kept rows than the suffix has
    assert lib.sdllm_validate_keep_idx(vp(4096), -1, 10, None) == sd.ERR_INVALID_ARG


def test_plans_do_not_depend_on_the_environment(lib):
    """A call's launch plan is a pure function of its parameters: the tuning variables earlier builds read
    from the environment change nothing."""
    import subprocess, sys
    code = ("import ctypes, paper_2601_17917_amd as sd\n"
            "p = sd.attn_params(sd.BF16, 8, 32, 32, 128, 1024, 2048, 32, 992, 32)\n"
            "pl = sd.plan_attention(p)\n"
            "u = sd.unmask_params(sd.BF16, 8, 32, 126464, 126464, 0.9, 0.3)\n"
            "print(pl.kv_splits, pl.rows_per_workgroup, pl.workgroups, sd.unmask_workspace_bytes(u))")
    outs = []
    for env in ({}, {"SDLLM_ATTN_RB": "2", "SDLLM_UNMASK_SPLITS": "3"}):
        r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True,
                           env={**os.environ, **env})
        assert r.returncode == 0, r.stderr
        outs.append(r.stdout)
    assert outs[0] == outs[1]


def test_noalloc_unmask_validates_and_rejects_sizes_beyond_its_scratch(lib):
    """The entry point that allocates nothing checks everything on the host before any HIP call: the same argument
    rules as sdllm_confidence_unmask, plus the limit of its device-resident scratch."""
    vp = ctypes.c_void_p
    ok = sd.unmask_params(sd.BF16, 8, 32, 126464, 126464, 0.9, 0.3)
    assert lib.sdllm_unmask_workspace_bytes(ctypes.byref(ok)) <= sd.NOALLOC_SCRATCH_BYTES
    args = [vp(4096), vp(4096), vp(4096), None, vp(4096), vp(4096), None, None]
    bad = list(args); bad[0] = None
    assert lib.sdllm_confidence_unmask_noalloc(ctypes.byref(ok), *bad) == sd.ERR_INVALID_ARG      # logits NULL
    bad = list(args); bad[0] = vp(4104)
    assert lib.sdllm_confidence_unmask_noalloc(ctypes.byref(ok), *bad) == sd.ERR_INVALID_ARG      # misaligned logits
    big = sd.unmask_params(sd.BF16, 64, 4096, 126464, 126464, 0.9, 0.3)       # 262144 rows: more triples than 1 MiB holds
    assert lib.sdllm_unmask_workspace_bytes(ctypes.byref(big)) > sd.NOALLOC_SCRATCH_BYTES
    assert lib.sdllm_confidence_unmask_noalloc(ctypes.byref(big), *args) == sd.ERR_UNSUPPORTED
    assert b"scratch" in lib.sdllm_last_error()


def test_probe_validation(lib):
    vp = ctypes.c_void_p
    assert lib.sdllm_probe_read(vp(4096), 0, vp(4096), None) == sd.ERR_INVALID_ARG
    assert lib.sdllm_probe_read(vp(4096), 24, vp(4096), None) == sd.ERR_INVALID_ARG          # not a multiple of 16
    assert lib.sdllm_probe_read(None, 32, vp(4096), None) == sd.ERR_INVALID_ARG
    assert lib.sdllm_probe_copy(vp(4096), vp(4104), 32, None) == sd.ERR_INVALID_ARG         # misaligned source
    assert lib.sdllm_probe_copy(None, vp(4096), 32, None) == sd.ERR_INVALID_ARG
    fl = ctypes.c_double(0.0)
    assert lib.sdllm_probe_mfma_bf16(0, 0, vp(4096), None, ctypes.byref(fl)) == sd.ERR_INVALID_ARG
    assert lib.sdllm_probe_mfma_bf16(10, 2, vp(4096), None, ctypes.byref(fl)) == sd.ERR_INVALID_ARG
    assert lib.sdllm_probe_mfma_bf16(10, 0, None, None, ctypes.byref(fl)) == sd.ERR_INVALID_ARG


@pytest.mark.parametrize("B,K,V,Hd", [(1, 1, 1, 32), (1, 32, 126464, 4096), (2, 32, 5000, 512), (3, 40, 777, 96),
                                       (8, 32, 126464, 4096), (16, 32, 152064, 3584), (9, 32, 700, 1024), (2, 32, 126464, 4096), (4, 32, 126464, 4096), (3, 32, 152064, 3584), (4, 32, 700, 64), (1, 32, 152064, 3584), (2, 32, 152064, 3584), (16, 4096, 100, 32)])
def test_lm_head_plan_is_consistent(lib, B, K, V, Hd):
    p = sd.lm_head_params(B, K, V, Hd, Hd, Hd, 0.9, 0.3)
    pl = sd.plan_lm_head(p)
    rows = B * K
    assert pl.rows_per_chunk in (32, 64, 128, 256)
    assert (pl.rows_per_chunk >= min(rows, 256)) and (rows > 32 or pl.rows_per_chunk == 32)
    assert pl.vocab_tiles * pl.vocab_rows_per_tile >= V > (pl.vocab_tiles - 1) * pl.vocab_rows_per_tile
    assert pl.row_chunks * pl.rows_per_chunk >= rows > (pl.row_chunks - 1) * pl.rows_per_chunk
    if rows <= 128:
        # stream shapes: 32-row sub-tiles per workgroup out of the compiled counts; one
        # workgroup per CU is resident, so the launch runs in rounds of 256 workgroups
        tt = pl.vocab_rows_per_tile // 32
        assert pl.vocab_rows_per_tile % 32 == 0
        assert tt in ((2, 4, 8, 12, 16, 20) if rows <= 32 else (2, 4, 8, 10, 12, 16) if rows <= 64 else (1, 2, 3, 4, 6, 8, 10, 16))
        assert pl.workgroups == pl.vocab_tiles and pl.row_chunks == 1
        rounds = -(-pl.vocab_tiles // 256)
        ideal = -(-V // 32) / 256.0                   # sub-tiles per CU if they could be spread evenly
        assert rounds * tt <= max(2.0, 1.35 * ideal + 2)
        if V == 126464:
            assert tt == 16                           # 247 workgroups
        if V == 152064:
            assert tt == (20 if rows <= 32 else 10)   # 238 workgroups in one round / 476 in two
    else:
        assert pl.vocab_rows_per_tile == 256
        assert pl.workgroups % 8 == 0 and pl.workgroups >= pl.vocab_tiles * pl.row_chunks
        assert pl.workgroups < pl.vocab_tiles * pl.row_chunks + 8 * pl.row_chunks
    assert pl.triples_per_position >= pl.vocab_tiles
    assert 64 * 1024 <= pl.lds_bytes <= 160 * 1024
    assert sd.lm_head_unmask_workspace_bytes(p) == rows * pl.triples_per_position * 12


def test_lm_head_packed_weight_host_side(lib):
    # size of the packed image: whole 16-row blocks x whole k-steps of one kilobyte each
    assert sd.lm_head_packed_weight_bytes(126464, 4096) == (126464 // 16) * (4096 // 32) * 1024
    assert sd.lm_head_packed_weight_bytes(17, 64) == 2 * 2 * 1024
    big = ctypes.c_size_t(-1).value
    assert lib.sdllm_lm_head_packed_weight_bytes(0, 64) == big and lib.sdllm_lm_head_packed_weight_bytes(5, 48) == big
    vp = ctypes.c_void_p
    assert lib.sdllm_lm_head_pack_weight(0, 64, 64, vp(4096), vp(8192), None) == sd.ERR_INVALID_ARG
    assert lib.sdllm_lm_head_pack_weight(10, 48, 64, vp(4096), vp(8192), None) == sd.ERR_INVALID_ARG
    assert lib.sdllm_lm_head_pack_weight(10, 64, 60, vp(4096), vp(8192), None) == sd.ERR_INVALID_ARG
    assert lib.sdllm_lm_head_pack_weight(10, 64, 64, None, vp(8192), None) == sd.ERR_INVALID_ARG
    assert lib.sdllm_lm_head_pack_weight(10, 64, 64, vp(4100), vp(8192), None) == sd.ERR_INVALID_ARG
    # the layout flag: only 0 and 1; a packed weight needs no row stride
    p = sd.lm_head_params(2, 32, 1000, 64, 64, 64, 0.9, 0.3, weight_packed=2)
    assert lib.sdllm_plan_lm_head(ctypes.byref(p), ctypes.byref(sd.LmHeadPlan())) == sd.ERR_INVALID_ARG
    p = sd.lm_head_params(2, 32, 1000, 64, 64, 0, 0.9, 0.3, weight_packed=1)
    assert lib.sdllm_plan_lm_head(ctypes.byref(p), ctypes.byref(sd.LmHeadPlan())) == 0
    p = sd.lm_head_params(2, 32, 1000, 64, 64, 0, 0.9, 0.3, weight_packed=0)
    assert lib.sdllm_plan_lm_head(ctypes.byref(p), ctypes.byref(sd.LmHeadPlan())) == sd.ERR_INVALID_ARG


@pytest.mark.parametrize("B,K,V", [(1, 32, 126464), (1, 32, 152064), (2, 32, 126464), (4, 32, 152064), (1, 8, 100),
                                   (3, 32, 5000), (9, 32, 700)])
def test_lm_head_plan_for_a_packed_weight(lib, B, K, V):
    p = sd.lm_head_params(B, K, V, 256, 256, 0, 0.9, 0.3, weight_packed=1)
    pl = sd.plan_lm_head(p)
    rows = B * K
    assert pl.vocab_tiles * pl.vocab_rows_per_tile >= V > (pl.vocab_tiles - 1) * pl.vocab_rows_per_tile
    if rows <= 32:
        assert pl.vocab_rows_per_tile // 64 in (1, 2, 4, 6, 8, 10) and pl.lds_bytes == 0   # operands straight from the image
        assert pl.vocab_rows_per_tile == {126464: 512, 152064: 640}.get(V, pl.vocab_rows_per_tile)
    elif rows <= 128:
        assert pl.vocab_rows_per_tile // 32 in (1, 2, 3, 4, 6, 8, 10, 16) and 64 * 1024 <= pl.lds_bytes <= 160 * 1024
    else:
        assert pl.vocab_rows_per_tile == 256
    assert pl.triples_per_position >= pl.vocab_tiles
    assert sd.lm_head_unmask_workspace_bytes(p) == rows * pl.triples_per_position * 12
