"""Checks on the compiled gfx950 code of the kernels (no GPU needed: hipcc cross-compiles).

The streaming-store hint on rows of C is easy to lose -- the compiler folds a hinted store with an
unhinted one on a sibling path and keeps neither hint -- and a change in register pressure can
push a kernel into scratch memory without any test of results noticing.  Both show in the
assembly."""
import os
import re
import subprocess

import pytest

from paper_2603_08734_amd import build as B


@pytest.fixture(scope="module")
def kernels_asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("isa") / "kernels.s"
    flags = [f for f in B.FLAGS if f not in ("-fPIC", "-shared")]
    src = os.path.join(B.CSRC, "kernels.hip")
    inc = os.path.join(B.HERE, "..", "include")
    subprocess.check_call([B.HIPCC, *flags, "-I", inc, "-S", "--cuda-device-only", "-o", str(out), src],
                          stderr=subprocess.DEVNULL)
    text = out.read_text()
    kernels = {}
    for chunk in re.split(r"\n\s*\.globl\s+", text)[1:]:
        name = chunk.split("\n", 1)[0].strip()
        end = chunk.find(".end_amdhsa_kernel")
        if end < 0:
            continue
        kernels[name] = chunk[:end]
    return kernels


def _stores(body):
    st = [l for l in body.splitlines() if "global_store_dwordx4" in l]
    return len(st), sum(" nt" in l for l in st)


def test_rows_of_c_leave_with_the_streaming_hint(kernels_asm):
    tile = {n: b for n, b in kernels_asm.items() if "rsh_tile_kernel" in n}
    irregular = {n: b for n, b in kernels_asm.items() if "rsh_irregular_kernel" in n}
    combine = {n: b for n, b in kernels_asm.items() if "rsh_combine_kernel" in n}
    # every kernel exists twice: fp32 sums (OutPlain) and the fused binary16 epilogue (OutFused);
    # the irregular kernel once more for a partial last feature panel
    assert len(tile) >= 60 and len(irregular) == 16 and len(combine) == 2
    for name, body in tile.items():
        n, nt = _stores(body)
        if "OutFused" in name:
            # scratch path: one ordinary store per 16-feature chunk; C path: the wave's 16 rows of
            # binary16 leave as 16 * (2 * chunks) 16-byte pieces, 64 per streaming store
            nch = int(re.search(r"rsh_tile_kernelILi(\d+)E", name).group(1))
            assert n - nt == nch and nt == max(1, nch // 2), f"{name}: {nt} streaming of {n} stores"
        else:
            assert n > 0 and nt * 2 == n, f"{name}: {nt} of {n} stores are streaming (C path streaming, scratch path ordinary)"
    for name, body in irregular.items():
        n, nt = _stores(body)
        assert n > 0 and nt == n, f"{name}: {nt} of {n} stores are streaming"
    for name, body in combine.items():
        st = [l for l in body.splitlines() if "global_store_dword" in l]
        want = "global_store_dwordx2" if "OutFused" in name else "global_store_dwordx4"
        assert st and all(want in l and " nt" in l for l in st), f"{name}: {st}"


def test_kernels_keep_their_registers(kernels_asm):
    for name, body in kernels_asm.items():
        m = re.search(r"\.amdhsa_private_segment_fixed_size\s+(\d+)", body)
        assert m, name
        spill = int(m.group(1))
        limit = 24 if "rsh_irregular_kernel" in name else 0     # a few registers of the 8-wave irregular kernel, outside its gather loops
        assert spill <= limit, f"{name} uses {spill} bytes of scratch per lane"


def test_tile_loop_waits_do_not_drain_global_loads(kernels_asm):
    """Inside the fragment loop of the 16-row tile kernels no wait may be vmcnt(0) together with
    outstanding prefetches: the generic fences did exactly that.  The loop is the code between the
    loop header label and its backward branch; it must contain MFMA and no `s_barrier`-less
    `vmcnt(0)` beyond the one that precedes staging of the single in-flight fragment."""
    name = next(n for n in kernels_asm if "rsh_tile_kernelILi8ELi4ELi2ELi32E" in n)   # 64-row windows, ring of two
    body = kernels_asm[name]
    loop = body[body.index("Inner Loop Header"):]
    loop = loop[:loop.index("s_endpgm")] if "s_endpgm" in loop else loop
    waits = re.findall(r"s_waitcnt vmcnt\((\d+)\)", loop[:loop.index("s_cbranch_scc")])
    assert waits and all(int(w) > 0 for w in waits), waits


def test_panel_kernels_use_the_32_row_mfma_and_transposing_reads(kernels_asm):
    """Windows of 128 or 256 rows: the product is formed by v_mfma_f32_32x32x16_f16 with the staged
    B tile read through the transposing LDS load, entries arrive as 16-byte loads, and rows of C
    leave as streaming 16-byte stores (partial sums as ordinary ones)."""
    panel = {n: b for n, b in kernels_asm.items() if "rsh_panel_kernel" in n}
    assert panel
    for name, body in panel.items():
        assert "v_mfma_f32_32x32x16_f16" in body and "ds_read_b64_tr_b16" in body, name
        assert "global_load_dwordx4" in body and "ds_write_b16" in body, name
        n, nt = _stores(body)   # each kernel holds both ends: rows of C (streaming) and partial sums (ordinary)
        if "OutPlain" in name:
            assert n > 0 and nt * 2 == n, f"{name}: {nt} of {n} stores are streaming"
        else:   # binary16 rows of C are half as wide
            assert any("global_store_dword" in l and " nt" in l for l in body.splitlines()), name
