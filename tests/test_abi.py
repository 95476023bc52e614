"""Host-side checks of the C ABI: the library loads, exports what include/roco.h declares, and rejects bad
arguments before launching anything (no GPU needed: every call here fails validation on the host)."""
import ctypes
import os
import re

import pytest

import paper_2402_06262_amd as roco

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EINVAL, EUNSUPPORTED, EWORKSPACE = -1, -2, -3


def declared_functions():
    text = open(os.path.join(ROOT, "include", "roco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(roco_[a-z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = roco.load_library()
    names = declared_functions()
    assert {"roco_prefill_compress", "roco_decode_step", "roco_prefill_workspace_bytes",
            "roco_decode_workspace_bytes", "roco_strerror", "roco_version", "roco_select_victims",
            "roco_probe_cache_read", "roco_profile_sampling", "roco_encode_block", "roco_block_workspace_bytes",
            "roco_decode_step_gqa", "roco_encode_block_gqa",
            "roco_select_retained", "roco_decode_step_launches", "roco_decode_step_static", "roco_set_overlap"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in roco.h but not exported"
    assert roco.roco_version() == 1
    assert roco.roco_strerror(0) == "success"
    assert "workspace" in roco.roco_strerror(EWORKSPACE)


def test_prefill_from_given_normalisers_validates_its_arguments():
    lib = roco.load_library()
    p = roco.RocoParams(4, 128, 64, 8, roco.ROCO_BF16)
    need = roco.prefill_workspace_bytes(p, 100)
    ok = 0x1000
    call = lambda lse, ws_bytes, group=1: lib.roco_prefill_compress_lse(
        ctypes.byref(p), group, ok, ok, ok, ok, 100, lse, ok, ok, ok, ok, ok, ok, ok, ws_bytes, None)
    assert call(None, need) == EINVAL          # the normalisers are the point of this entry
    assert call(0x1004, need) == EINVAL        # misaligned
    assert call(ok, need - 1) == EWORKSPACE
    assert call(ok, need, group=0) == EINVAL
    assert call(ok, need, group=65) == EUNSUPPORTED


def test_mfma_probe_arguments_are_validated_on_the_host():
    lib = roco.load_library()
    assert lib.roco_probe_mfma(0, 16, 0, 0x1000, 1 << 20, None) == EINVAL
    assert lib.roco_probe_mfma(16, 0, 0, 0x1000, 1 << 20, None) == EINVAL
    assert lib.roco_probe_mfma(16, 16, 4, 0x1000, 1 << 20, None) == EINVAL
    assert lib.roco_probe_mfma(16, 16, -1, 0x1000, 1 << 20, None) == EINVAL
    assert lib.roco_probe_mfma(16, 16, 1, None, 1 << 20, None) == EINVAL
    assert lib.roco_probe_mfma(16, 16, 1, 0x1000, 16 * 1024 - 1, None) == EWORKSPACE


def test_params_struct_layout_matches_the_header():
    assert ctypes.sizeof(roco.RocoParams) == 44
    names = [f[0] for f in roco.RocoParams._fields_]
    assert names == ["units", "head_dim", "budget", "scope", "dtype", "scale", "recency_window", "recency_bias",
                     "importance", "scope_kind", "sinks"]
    # the header declares the same members in the same order
    text = open(os.path.join(ROOT, "include", "roco.h")).read()
    body = re.sub(r"/\*.*?\*/", "", text[text.index("typedef struct roco_params"):text.index("} roco_params;")], flags=re.S)
    assert re.findall(r"\b(?:int32_t|float)\s+(\w+)\s*;", body) == names


def test_policy_fields_are_validated():
    ok = roco.RocoParams(8, 128, 256, 16, roco.ROCO_BF16, importance=roco.ROCO_IMPORTANCE_OLDEST,
                         scope_kind=roco.ROCO_SCOPE_ALL, sinks=4)
    assert roco.decode_workspace_bytes(ok) > 0
    for bad in (dict(importance=5), dict(importance=-1), dict(scope_kind=3), dict(sinks=-1),
                dict(importance=roco.ROCO_IMPORTANCE_LAST, scope_kind=roco.ROCO_SCOPE_STD),
                dict(importance=roco.ROCO_IMPORTANCE_COUNT, scope_kind=roco.ROCO_SCOPE_STD)):
        assert roco.decode_workspace_bytes(roco.RocoParams(8, 128, 256, 16, roco.ROCO_BF16, **bad)) == 0
    lib = roco.load_library()
    need = roco.decode_workspace_bytes(ok)
    # a policy that ranks by position needs pos
    assert lib.roco_select_victims(ctypes.byref(ok), 0x1000, None, 0x1000, 0x1000, 0x1000, need, None) == EINVAL


def test_workspace_queries():
    p = roco.RocoParams(512, 128, 2048, 64, roco.ROCO_BF16)
    assert roco.decode_workspace_bytes(p) >= 512 * 2048 * 4
    assert roco.prefill_workspace_bytes(p, 3072) >= 512 * 3072 * 4 * 4
    assert roco.prefill_workspace_bytes(p, 0) == 0
    assert roco.decode_workspace_bytes(roco.RocoParams(4, 96, 128, 16, roco.ROCO_F32)) == 0  # head_dim
    assert roco.decode_workspace_bytes(roco.RocoParams(4, 64, 128, 129, roco.ROCO_F32)) == 0  # scope > B
    assert roco.decode_workspace_bytes(roco.RocoParams(65535, 64, 128, 16, roco.ROCO_F32)) > 0
    assert roco.decode_workspace_bytes(roco.RocoParams(65536, 64, 128, 16, roco.ROCO_F32)) == 0  # units per call
    # which decode shape a call takes: fused from 128 units on while the budget fits LDS, else the split pair
    assert roco.decode_step_launches(roco.RocoParams(512, 128, 2048, 64, roco.ROCO_BF16)) == 1
    assert roco.decode_step_launches(roco.RocoParams(40, 128, 4096, 64, roco.ROCO_BF16)) == 2
    assert roco.decode_step_launches(roco.RocoParams(127, 128, 2048, 64, roco.ROCO_BF16)) == 2
    assert roco.decode_step_launches(roco.RocoParams(128, 128, 2048, 64, roco.ROCO_BF16)) == 1
    assert roco.decode_step_launches(roco.RocoParams(512, 128, 8192, 64, roco.ROCO_BF16)) == 2
    assert roco.load_library().roco_decode_step_launches(ctypes.byref(roco.RocoParams(4, 96, 128, 16, roco.ROCO_F32))) == EUNSUPPORTED


def _decode(p, ptrs=None, ws_bytes=1 << 30):
    lib = roco.load_library()
    a = [0x1000] * 14 if ptrs is None else ptrs
    return lib.roco_decode_step(ctypes.byref(p), *a[:14], ws_bytes, None)


def _prefill(p, L_max=64, ptrs=None, ws_bytes=1 << 30):
    lib = roco.load_library()
    a = [0x1000] * 12 if ptrs is None else ptrs
    return lib.roco_prefill_compress(ctypes.byref(p), a[0], a[1], a[2], a[3], L_max, *a[4:12], ws_bytes, None)


@pytest.mark.parametrize("kw,code", [
    (dict(units=0), EINVAL), (dict(budget=0), EINVAL), (dict(scope=0), EINVAL), (dict(scope=129), EINVAL),
    (dict(recency_window=-1), EINVAL), (dict(head_dim=96), EUNSUPPORTED), (dict(dtype=7), EUNSUPPORTED),
    (dict(scale=float("nan")), EINVAL),
])
def test_invalid_params_are_rejected_on_the_host(kw, code):
    base = dict(units=4, head_dim=64, budget=128, scope=16, dtype=roco.ROCO_F32)
    base.update(kw)
    p = roco.RocoParams(**base)
    assert _decode(p) == code
    assert _prefill(p) == code


def test_null_misaligned_and_small_workspace_are_rejected_on_the_host():
    p = roco.RocoParams(4, 64, 128, 16, roco.ROCO_F32)
    lib = roco.load_library()
    assert lib.roco_decode_step(None, *([0x1000] * 14), 1 << 30, None) == EINVAL
    for bad in range(12):  # the twelve required pointers (evicted_* are optional)
        ptrs = [0x1000] * 14
        order = [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 13]
        ptrs[order[bad]] = None
        assert _decode(p, ptrs) == EINVAL
        ptrs[order[bad]] = 0x1004
        assert _decode(p, ptrs) == EINVAL
    assert _decode(p, ws_bytes=roco.decode_workspace_bytes(p) - 1) == EWORKSPACE
    for bad in [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 11]:  # O (index 10) may be NULL
        ptrs = [0x1000] * 12
        ptrs[bad] = None
        assert _prefill(p, ptrs=ptrs) == EINVAL
    assert _prefill(p, L_max=0) == EINVAL
    assert _prefill(p, L_max=64, ws_bytes=roco.prefill_workspace_bytes(p, 64) - 1) == EWORKSPACE


def test_encode_block_validates_on_the_host():
    EUNS = EUNSUPPORTED
    lib = roco.load_library()
    p = roco.RocoParams(4, 128, 256, 16, roco.ROCO_BF16)
    need = roco.block_workspace_bytes(p, 8)
    assert need > 4 * 64 * 256 * 4  # logits of 64 query rows per unit, whatever the block
    args = [0x1000] * 14

    def call(params, block, a=args, ws=need):
        r1 = lib.roco_encode_block(ctypes.byref(params), block, *a[:14], ws, None)
        r2 = lib.roco_encode_block_gqa(ctypes.byref(params), block, 1, *a[:14], ws, None)  # one head: same checks
        assert r1 == r2
        return r1

    def grouped(block, group):
        return (lib.roco_encode_block_gqa(ctypes.byref(p), block, group, *args, need, None),
                lib.roco_decode_step_gqa(ctypes.byref(p), group, *args, need, None))

    assert grouped(1, 0) == (EINVAL, EINVAL) and grouped(1, 65) == (EUNS, EUNS)
    assert grouped(13, 5)[0] == EUNS and grouped(17, 4)[0] == EUNS  # more than 64 query rows

    assert call(p, 0) == EINVAL and call(p, 257) == EINVAL
    assert call(p, 65) == EUNS
    assert call(roco.RocoParams(4, 96, 256, 16, roco.ROCO_BF16), 4) == EUNS  # head_dim
    assert call(roco.RocoParams(4, 128, 254, 16, roco.ROCO_BF16), 4) == EUNS  # budget not a multiple of 4
    assert roco.block_workspace_bytes(roco.RocoParams(4, 96, 256, 16, roco.ROCO_BF16), 4) == 0
    assert roco.block_workspace_bytes(roco.RocoParams(4, 64, 256, 16, roco.ROCO_F32), 4) > 0  # every dtype / head_dim
    assert call(p, 8, ws=need - 1) == EWORKSPACE
    for bad in [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 13]:  # evicted_slot / evicted_pos (11, 12) may be NULL
        a = list(args)
        a[bad] = None
        assert call(p, 8, a) == EINVAL


def test_select_retained_validates_on_the_host():
    lib = roco.load_library()
    p = roco.RocoParams(4, 128, 256, 16, roco.ROCO_BF16)
    need = roco.decode_workspace_bytes(p)

    def call(params, keep, stats=0x1000, pos=0x1000, n_used=0x1000, mask=0x1000, ws=0x1000, nbytes=need):
        return lib.roco_select_retained(ctypes.byref(params), keep, stats, pos, n_used, mask, ws, nbytes, None)

    assert call(p, -1) == EINVAL
    assert call(p, 10, nbytes=need - 1) == EWORKSPACE
    assert call(p, 10, stats=None) == EINVAL and call(p, 10, n_used=None) == EINVAL and call(p, 10, mask=None) == EINVAL
    assert call(p, 10, mask=0x1004) == EINVAL  # misaligned
    window = roco.RocoParams(4, 128, 256, 16, roco.ROCO_BF16, scope_kind=roco.ROCO_SCOPE_WINDOW)
    assert call(window, 10, pos=None) == EINVAL  # this policy ranks by position
    assert call(roco.RocoParams(4, 96, 256, 16, roco.ROCO_BF16), 10) == EUNSUPPORTED


def test_loading_fails_loudly_when_the_library_is_missing(monkeypatch):
    from paper_2402_06262_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_NAME", "libroco_missing.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load_library()


def test_static_scratch_decode_step_validates_on_the_host():
    """Argument errors and shapes beyond the static scratch are reported before any HIP call."""
    lib = roco.load_library()
    ok = roco.RocoParams(4, 128, 64, 8, roco.ROCO_BF16)
    args = [0x1000] * 13
    assert lib.roco_decode_step_static(None, *args, None) == EINVAL
    assert lib.roco_decode_step_static(ctypes.byref(ok), None, *args[1:], None) == EINVAL
    assert lib.roco_decode_step_static(ctypes.byref(ok), 0x1001, *args[1:], None) == EINVAL
    big = roco.RocoParams(4096, 128, 4096, 64, roco.ROCO_BF16)
    assert roco.decode_workspace_bytes(big) > 32 << 20
    assert lib.roco_decode_step_static(ctypes.byref(big), *args, None) == -5
    assert "static" in roco.roco_strerror(-5)


def test_set_overlap_validates_on_the_host():
    lib = roco.load_library()
    ok = [4, 16, 0x1000, None, 0x1000, 16, 0x1000, None, 0x1000, 64, 0x1000, 0x1000, None]
    bad_units, bad_max, big_max, misaligned = list(ok), list(ok), list(ok), list(ok)
    bad_units[0] = 0
    bad_max[9] = 0
    big_max[9] = (1 << 19) + 1
    misaligned[3] = 0x1004
    assert lib.roco_set_overlap(*bad_units) == EINVAL
    assert lib.roco_set_overlap(*bad_max) == EINVAL
    assert lib.roco_set_overlap(*big_max) == EUNSUPPORTED
    assert lib.roco_set_overlap(*misaligned) == EINVAL
    no_out = list(ok)
    no_out[10] = None
    assert lib.roco_set_overlap(*no_out) == EINVAL


def test_header_is_plain_c_and_a_c_program_links_against_the_library(tmp_path):
    """include/roco.h compiles as C99 with warnings as errors; a C program calls the host-only entry points (sizes,
    codes, argument validation: nothing is launched) through the shared library."""
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_roco.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "roco.h"
int main(void) {
  roco_params p;
  memset(&p, 0, sizeof p);
  p.units = 4; p.head_dim = 128; p.budget = 256; p.scope = 16; p.dtype = ROCO_BF16;
  if (sizeof(roco_params) != 44) return 1;
  if (roco_version() != ROCO_VERSION) return 2;
  if (roco_decode_workspace_bytes(&p) == 0 || roco_prefill_workspace_bytes(&p, 512) == 0) return 3;
  if (roco_block_workspace_bytes(&p, 8) == 0) return 4;
  p.head_dim = 96;
  if (roco_decode_workspace_bytes(&p) != 0) return 5;
  p.head_dim = 128;
  /* null pointers are refused on the host, before anything is launched */
  if (roco_decode_step(&p, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) != ROCO_EINVAL) return 6;
  if (roco_set_overlap(0, 1, NULL, NULL, NULL, 1, NULL, NULL, NULL, 1, NULL, NULL, NULL) != ROCO_EINVAL) return 7;
  if (strcmp(roco_strerror(ROCO_OK), "success") != 0) return 8;
  printf("ok %d\n", roco_decode_step_launches(&p));
  return 0;
}
''')
    exe = tmp_path / "use_roco"
    lib_dir = os.path.dirname(roco.binding.library_path())
    cmd = [cc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src),
           "-L", lib_dir, "-l:libroco.so", f"-Wl,-rpath,{lib_dir}", "-o", str(exe)]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, (run.returncode, run.stdout, run.stderr)
    assert run.stdout.startswith("ok ")
