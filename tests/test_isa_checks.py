"""Checks on the gfx950 assembly hipcc generates for the library's own kernels
(compiled here with --save-temps; needs no GPU).

Each check guards something that went wrong once or is ruled out on the
target machines:
  * no scalar register left undefined on a path ("implicit-def: $sgpr"): a
    pointer selected by a three-way uniform branch once compiled to code that
    left the destination pointer unset on one path, and the store went wild;
  * no scratch memory (register spills) in any kernel;
  * no packed-fp32 arithmetic (the build disables it; the adds of the
    reduction must stay single IEEE binary32 operations);
  * no write through the scalar data cache;
  * the streaming kernels keep their 16-byte vector accesses.
"""
import os
import re
import subprocess

import pytest

from paper_2602_06499_amd import build

KERNELS = os.path.join(build.CSRC, "fcdp_kernels.hip")


@pytest.fixture(scope="module")
def asm(tmp_path_factory):
    d = tmp_path_factory.mktemp("isa")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    subprocess.check_call([hipcc, *flags, "--save-temps", "-c", "-x", "hip", KERNELS,
                           "-o", str(d / "kernels.o")], cwd=str(d),
                          stderr=subprocess.DEVNULL)
    files = [f for f in os.listdir(d) if f.endswith(".s") and "gfx950" in f]
    assert len(files) == 1, files
    text = open(d / files[0]).read()
    kernels = {}
    for m in re.finditer(r"^(_Z\w+):.*?\.end_amdhsa_kernel", text, flags=re.S | re.M):
        kernels[m.group(1)] = m.group(0)
    assert len(kernels) > 50
    return kernels


def _named(kernels, part):
    return {k: v for k, v in kernels.items() if part in k}


def test_no_scalar_register_is_left_undefined(asm):
    bad = [k for k, body in asm.items() if "implicit-def: $sgpr" in body]
    assert not bad, bad


def test_no_scratch_no_packed_fp32_no_scalar_cache_writes(asm):
    scalar_writes = re.compile(r"^\s*(s_store_|s_buffer_store_|s_scratch_store_|s_atomic_|"
                               r"s_buffer_atomic_|s_dcache_wb|s_dcache_inv)", re.M)
    for name, body in asm.items():
        assert ".amdhsa_private_segment_fixed_size 0" in body, name
        assert ".amdhsa_uses_dynamic_stack 0" in body, name
        assert "scratch_" not in body.split(".amdhsa_kernel")[0], name
        assert not re.search(r"v_pk_(add|mul|fma)_f32", body), name
        assert not scalar_writes.search(body), name


def test_streaming_kernels_keep_their_vector_width(asm):
    copies = _named(asm, "copy_pieces")
    reduces = _named(asm, "reduce_ranks")
    assert len(copies) == 16 and len(reduces) == 64
    for name, body in copies.items():
        assert "global_load_dwordx4" in body and "global_store_dwordx4" in body, name
    for name, body in reduces.items():
        assert "global_load_dwordx4" in body or "global_load_dwordx2" in body, name
        assert "v_add_f32" in body and "v_fma" not in body and "v_mac" not in body, name
        m = re.search(r"\.amdhsa_next_free_vgpr (\d+)", body)
        assert m and int(m.group(1)) <= 256, (name, m and m.group(1))   # at least 2 waves per SIMD
