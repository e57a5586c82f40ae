"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, and rejects bad arguments before any device work."""
import ctypes
import json
import struct
import os
import re

import numpy as np
import pytest

from paper_2509_23410_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    src = open(os.path.join(ROOT, "include", "patch.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(patch_[a-z0-9_]+)\s*\(", src)))


def test_header_symbols_are_exported():
    names = header_functions()
    assert "patch_pack" in names and "patch_gemm" in names and len(names) >= 12
    L = B.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared in patch.h but not exported"
    assert sorted(B.EXPORTS) == names


def test_strerror_and_version():
    assert B.strerror(B.OK) == "ok"
    assert "2:4" in B.strerror(B.ERR_NOT_24)
    assert "gfx950" in B.version()


def test_argument_errors_without_device():
    L = B.lib()
    tm = np.ones((2, 2), np.uint8)
    out = ctypes.c_void_p(0)
    fake = 0x1000  # never dereferenced: all of these fail on the host first
    assert L.patch_pack(0, 128, 128, tm.ctypes.data, 64, 0, ctypes.byref(out)) == B.ERR_ARG
    assert L.patch_pack(fake, 128, 128, 0, 64, 0, ctypes.byref(out)) == B.ERR_ARG
    assert L.patch_pack(fake, -1, 128, tm.ctypes.data, 64, 0, ctypes.byref(out)) == B.ERR_ARG
    assert L.patch_pack(fake, 128, 128, tm.ctypes.data, 32, 0, ctypes.byref(out)) == B.ERR_SHAPE
    assert L.patch_pack(fake, 100, 128, tm.ctypes.data, 64, 0, ctypes.byref(out)) == B.ERR_SHAPE
    assert L.patch_pack(fake + 2, 128, 128, tm.ctypes.data, 64, 0, ctypes.byref(out)) == B.ERR_ARG  # misaligned
    assert out.value is None
    assert L.patch_gemm(fake, 1, 0, fake, 0) == B.ERR_ARG
    two = (ctypes.c_void_p * 2)(0, 0)
    assert L.patch_gemm_many(fake, 1, two, two, 2, 0, None) == B.ERR_ARG   # null handles
    assert L.patch_gemm_many(fake, 1, two, two, 0, 0, None) == B.ERR_ARG   # count out of range
    assert L.patch_gemm_many(fake, 1, two, two, 9, 0, None) == B.ERR_ARG
    assert L.patch_gemm(0, 1, fake, fake, 0) == B.ERR_ARG
    assert L.patch_apply_mask(fake, fake, tm.ctypes.data, 128, 128, 48, fake, 0) == B.ERR_SHAPE
    assert L.patch_hard_masks(None, fake, 128, 128, 64, tm.ctypes.data, fake, 0) == B.ERR_ARG
    assert L.patch_hard_masks(fake, fake, 128, 100, 64, tm.ctypes.data, fake, 0) == B.ERR_SHAPE
    assert L.patch_hard_masks(fake, fake + 2, 128, 128, 64, tm.ctypes.data, fake, 0) == B.ERR_ARG
    assert L.patch_unpack(0, fake, 0) == B.ERR_ARG
    assert L.patch_packed_bytes(0) == 0
    assert L.patch_gemm_workspace_bytes(256, 0, None) == 0
    assert L.patch_tune(fake, 1, 0, fake, None, 0, None, 5, None, None) == B.ERR_ARG
    assert L.patch_tune_all(fake, 1, 0, fake, None, 0, None, 5, None, 0, None) == B.ERR_ARG
    assert L.patch_gemm_static(fake, 1, 0, fake, 0) == B.ERR_ARG
    assert L.patch_probe_matrix_rate(4, fake, 1 << 20, 1, 1, fake, 1 << 20, 0) == B.ERR_ARG
    assert L.patch_probe_stream_read(fake, 1024, 1, 100, fake, 1 << 20, 0) == B.ERR_ARG
    assert L.patch_probe_lds_fill(5, fake, 1 << 20, 1, 1, fake, 1 << 20, 0) == B.ERR_ARG
    assert L.patch_probe_lds_fill(0, fake, 1000, 1, 1, fake, 1 << 20, 0) == B.ERR_SIZE        # less than one 48 KB chunk
    assert L.patch_probe_lds_fill(0, fake, 1 << 20, 4, 1, fake, 1024, 0) == B.ERR_SIZE        # out too small
    assert L.patch_probe_lds_read(0, 10, fake, 1 << 20, 0) == B.ERR_ARG
    assert L.patch_probe_lds_read(4, 10, fake, 4 * 256 * 4 - 1, 0) == B.ERR_SIZE              # out too small
    assert L.patch_probe_store_tiles(2, 0, fake, 1 << 30, 256, 256, 0) == B.ERR_ARG           # no such pattern
    assert L.patch_probe_store_tiles(0, 0, fake, 1 << 30, 256, 300, 0) == B.ERR_ARG           # N not a multiple of 256
    assert L.patch_probe_store_tiles(0, 0, fake, 256 * 256 * 4 - 1, 256, 256, 0) == B.ERR_SIZE  # Y smaller than M x N fp32
    assert L.patch_probe_store_tiles(1, 1, fake, 256 * 512 * 2 - 1, 256, 512, 0) == B.ERR_SIZE  # ... than M x N bf16
    # 4-bit storage
    assert L.patch_pack4(0, 128, 128, tm.ctypes.data, 64, 0, ctypes.byref(out)) == B.ERR_ARG
    assert L.patch_gemm4_ex(fake, 1, 0, fake, None, 0, 0) == B.ERR_ARG
    assert L.patch_gemm4_ex(None, 1, fake, fake, None, 0, 0) == B.ERR_ARG
    assert L.patch_pack4(fake, 128, 128, 0, 64, 0, ctypes.byref(out)) == B.ERR_ARG
    assert L.patch_pack4(fake, 128, 128, tm.ctypes.data, 64, 0, None) == B.ERR_ARG
    assert L.patch_pack4(fake, 128, 128, tm.ctypes.data, 32, 0, ctypes.byref(out)) == B.ERR_SHAPE
    assert L.patch_pack4(fake, 128, 100, tm.ctypes.data, 64, 0, ctypes.byref(out)) == B.ERR_SHAPE
    assert L.patch_pack4(fake + 2, 128, 128, tm.ctypes.data, 64, 0, ctypes.byref(out)) == B.ERR_ARG  # misaligned
    assert out.value is None
    assert L.patch_gemm4(fake, 1, 0, fake, 0) == B.ERR_ARG
    assert L.patch_gemm4(0, 1, fake, fake, 0) == B.ERR_ARG
    assert L.patch_gemm4(fake, -1, fake, fake, 0) == B.ERR_ARG
    assert L.patch_gemm4_many(fake, 1, two, two, 2, 0) == B.ERR_ARG   # null handles
    assert L.patch_gemm4_many(fake, 1, two, two, 0, 0) == B.ERR_ARG   # count out of range
    assert L.patch_gemm4_many(fake, 1, two, two, 9, 0) == B.ERR_ARG
    assert L.patch_unpack4(0, fake, None, None, 0) == B.ERR_ARG
    assert L.patch_pack_from4(0, 0, ctypes.byref(out)) == B.ERR_ARG
    assert L.patch_pack_from4(fake, 0, None) == B.ERR_ARG
    assert L.patch_packed4_bytes(0) == 0
    assert L.patch_packed4_dims(0, None, None, None, None) == B.ERR_ARG
    L.patch_free4(0)
    L.patch_free(0)
    with pytest.raises(B.PatchError):
        B.patch_pack4(fake, 128, 128, np.ones(3, np.uint8), 64)
    with pytest.raises(B.PatchError):
        B.patch_pack(fake, 128, 128, np.ones(3, np.uint8), 64)


def _fnv1a(data: bytes, h: int = 14695981039346656037) -> int:
    for b in data:
        h = ((h ^ b) * 1099511628211) & 0xFFFFFFFFFFFFFFFF
    return h


def _saved(magic=b"PATCHPK\0", layout=1, tile=64, N=128, K=128, map_bytes=4, payload=b"\0" * 4 * 8192, aux=b"", tm=b"\1\1\1\1",
           checksum=None, claim_payload=None):
    """A saved-weight buffer written by hand from the documented format: 64-byte header, tile map, payload (and the
    scales of the 4-bit storage), each part at a multiple of 64 bytes."""
    pad = lambda b: b + b"\0" * (-len(b) % 64)
    body = pad(tm) + (pad(payload) if aux else payload) + aux
    cs = _fnv1a(aux, _fnv1a(payload, _fnv1a(tm))) if checksum is None else checksum
    head = struct.pack("<8sIIqqQQQQ", magic, layout, tile, N, K, map_bytes, len(payload) if claim_payload is None else claim_payload,
                       len(aux), cs)
    assert len(head) == 64
    return np.frombuffer(head + body, np.uint8).copy()


def test_saved_weight_is_checked_on_the_host():
    """patch_deserialize / patch_deserialize4 refuse, before any device work, everything that is not a buffer the
    library wrote: wrong magic or layout number, impossible shapes, sizes that disagree with the tile map or with the
    buffer, map entries other than 0 / 1, a checksum that does not match."""
    L = B.lib()
    out = ctypes.c_void_p(0)
    assert L.patch_serialized_bytes(0) == 0 and L.patch_serialized4_bytes(0) == 0
    fake = 0x1000
    assert L.patch_serialize(0, fake, 1 << 20, 0) == B.ERR_ARG
    assert L.patch_serialize(fake, 0, 1 << 20, 0) == B.ERR_ARG
    assert L.patch_serialize4(0, fake, 1 << 20, 0) == B.ERR_ARG
    for name, magic in (("patch_deserialize", b"PATCHPK\0"), ("patch_deserialize4", b"PATCHQ4\0")):
        fn = getattr(L, name)
        other = b"PATCHQ4\0" if name == "patch_deserialize" else b"PATCHPK\0"
        aux = b"\0" * (128 * 2 * 2) if name == "patch_deserialize4" else b""
        call = lambda a, n=None: fn(a.ctypes.data, a.size if n is None else n, 0, ctypes.byref(out))
        assert fn(0, 64, 0, ctypes.byref(out)) == B.ERR_ARG
        good = _saved(magic=magic, aux=aux)
        assert fn(good.ctypes.data, good.size, 0, None) == B.ERR_ARG
        assert call(good, 63) == B.ERR_SIZE                                       # shorter than a header
        assert call(_saved(magic=other, aux=aux)) == B.ERR_ARG                     # the other storage's buffer
        assert call(_saved(magic=b"NOTPATCH", aux=aux)) == B.ERR_ARG
        assert call(_saved(magic=magic, layout=2, aux=aux)) == B.ERR_ARG          # written by another layout
        assert call(_saved(magic=magic, tile=32, aux=aux)) == B.ERR_SHAPE
        assert call(_saved(magic=magic, N=100, aux=aux)) == B.ERR_SHAPE
        assert call(_saved(magic=magic, N=-128, aux=aux)) == B.ERR_ARG
        assert call(_saved(magic=magic, map_bytes=5, aux=aux)) == B.ERR_ARG       # not (N / tile) (K / tile)
        assert call(good, good.size - 1) == B.ERR_SIZE                            # truncated
        assert call(_saved(magic=magic, aux=aux, claim_payload=1 << 40)) == B.ERR_SIZE
        assert call(_saved(magic=magic, aux=aux, tm=b"\1\2\1\1")) == B.ERR_ARG    # a map entry that is neither 0 nor 1
        assert call(_saved(magic=magic, aux=aux, checksum=12345)) == B.ERR_ARG
        flipped = good.copy()
        flipped[-1] ^= 1
        assert call(flipped) == B.ERR_ARG                                         # one bit of the last byte
    assert call is not None and out.value is None


def test_tune_table_host_logic():
    """The table of tuned schedules is host memory only: buckets, put / get / replace, misses, the workspace rule."""
    assert [B.tune_bucket(m) for m in (1, 2, 3, 4, 5, 16, 17, 512, 513, 4096)] == [1, 2, 4, 4, 8, 16, 32, 512, 1024, 4096]
    tab = B.TuneTable()
    assert len(tab) == 0 and tab.get(1, 4096, 4096, 128, 512) is None
    tab.put(1, 4096, 4096, 128, 512, path=B.PATH_DECODE, split_k=8, variant=3)
    tab.put(3000, 4096, 4096, 128, 512, path=B.PATH_PREFILL, split_k=1, variant=0)
    tab.put(40, 4096, 4096, 128, 512, path=B.PATH_DECODE, split_k=4, variant=4, uses_workspace=True)
    assert len(tab) == 3
    assert tab.get(1, 4096, 4096, 128, 512) == dict(path=B.PATH_DECODE, split_k=8, variant=3, uses_workspace=False)
    assert tab.get(4096, 4096, 4096, 128, 512)["path"] == B.PATH_PREFILL        # 3000 and 4096 share the bucket
    assert tab.get(2048, 4096, 4096, 128, 512) is None                           # another bucket
    assert tab.get(1, 4096, 4096, 128, 511) is None and tab.get(1, 4096, 4096, 64, 512) is None   # another map / tile
    assert tab.get(40, 4096, 4096, 128, 512) is None                             # stored with a workspace, none given
    got = tab.get(40, 4096, 4096, 128, 512, workspace=0x1000, workspace_bytes=1 << 20)
    assert got == dict(path=B.PATH_DECODE, split_k=4, variant=4, uses_workspace=True)
    tab.put(1, 4096, 4096, 128, 512, path=B.PATH_DECODE, split_k=2, variant=2)   # replace
    assert len(tab) == 3 and tab.get(1, 4096, 4096, 128, 512)["split_k"] == 2
    L = B.lib()
    o = B.GemmOpts()
    assert L.patch_tune_table_get(tab.handle, 0, 4096, 4096, 128, 512, None, 0, ctypes.byref(o)) == B.ERR_ARG      # M < 1
    assert L.patch_tune_table_get(tab.handle, 1, 4096, 4000, 128, 512, None, 0, ctypes.byref(o)) == B.ERR_ARG      # K % tile
    assert L.patch_tune_table_get(tab.handle, 1, 4096, 4096, 128, 5000, None, 0, ctypes.byref(o)) == B.ERR_ARG     # more 2:4 tiles than tiles
    bad = B.GemmOpts(7, 0, 0, None, 0, 0)
    assert L.patch_tune_table_put(tab.handle, 1, 4096, 4096, 128, 512, ctypes.byref(bad)) == B.ERR_ARG
    assert L.patch_tune_table_create(None) == B.ERR_ARG and L.patch_tune_table_size(None) == 0
    assert L.patch_tune_layer(None, 0x1000, 1, 0x1000, 64, None, 0x1000, None, 0, None, 3) == B.ERR_ARG
    # export / import: plain records, all or nothing
    saved = tab.export()
    assert len(saved) == 3 and {e["m_bucket"] for e in saved} == {1, 64, 4096}
    assert all(e["N"] == 4096 and e["K"] == 4096 and e["tile"] == 128 and e["n_sparse_tiles"] == 512 for e in saved)
    assert json.loads(json.dumps(saved)) == saved
    other = B.TuneTable()
    other.put(1, 4096, 4096, 128, 512, path=B.PATH_PREFILL)                     # replaced by the import
    other.put(7, 896, 896, 128, 10, path=B.PATH_DECODE)                          # kept
    other.load(saved)
    assert len(other) == 4 and other.get(1, 4096, 4096, 128, 512) == tab.get(1, 4096, 4096, 128, 512)
    assert other.get(40, 4096, 4096, 128, 512, workspace=0x1000, workspace_bytes=64) == got
    assert other.get(40, 4096, 4096, 128, 512) is None and other.get(7, 896, 896, 128, 10)["path"] == B.PATH_DECODE
    for field, value in (("m_bucket", 3), ("m_bucket", 0), ("K", 4000), ("tile", 32), ("n_sparse_tiles", 5000), ("path", 9), ("split_k", 17), ("variant", -1)):
        broken = [dict(e) for e in saved]
        broken[2][field] = value
        fresh = B.TuneTable()
        with pytest.raises(B.PatchError) as err:
            fresh.load(broken)
        assert err.value.status == B.ERR_ARG and len(fresh) == 0, field       # the two good records before it were not stored
        fresh.close()
    n = ctypes.c_size_t(99)
    small = (B.TuneEntry * 2)()
    assert L.patch_tune_table_export(tab.handle, small, 2, ctypes.byref(n)) == B.ERR_SIZE and n.value == 3
    assert L.patch_tune_table_export(tab.handle, None, 2, ctypes.byref(n)) == B.ERR_ARG
    assert L.patch_tune_table_export(None, small, 2, ctypes.byref(n)) == B.ERR_ARG
    assert L.patch_tune_table_export(tab.handle, small, 2, None) == B.ERR_ARG
    assert L.patch_tune_table_import(None, small, 0) == B.ERR_ARG and L.patch_tune_table_import(tab.handle, None, 1) == B.ERR_ARG
    assert L.patch_tune_table_import(tab.handle, None, 0) == B.OK and len(tab) == 3
    other.close()
    tab.close()


def test_wreg_kernel_keeps_named_registers_to_itself(tmp_path):
    """prefill_kernel_wreg addresses a[0:255] and v[64:251] by name inside its asm statements (the whole step loop is one
    statement); between those statements weight loads, LDS reads and LDS-DMA are in flight into these registers, so the
    code the compiler generates around them must not touch them, nor m0 (written by the asm for LDS-DMA), and must not
    spill a vector register (a spill could move a value the asm owns).  The scalar registers the loop names (s74 - s97)
    are initialised and consumed inside the one loop statement, which declares them clobbered: the compiler may use them
    elsewhere.  v252 - v255 belong to nobody.  Every instantiation is checked."""
    import re
    from paper_2509_23410_amd import build
    text = open(build.device_asm("gemm_prefill_wreg.hip", str(tmp_path / "wreg.s"))).read()
    bodies = list(re.finditer(r"^(_ZN5patch19prefill_kernel_wreg\w*):[^\n]*\n(.*?)^\.Lfunc_end\d+:", text, re.S | re.M))
    assert len(bodies) == 3, "expected the instantiations <0>, <1>, <2>"
    for m in bodies:
        name = m.group(1)
        inasm, n_asm = False, 0
        for line in m.group(2).splitlines():
            if "#ASMSTART" in line:
                inasm, n_asm = True, n_asm + 1
                continue
            if "#ASMEND" in line:
                inasm = False
                continue
            code = line.split(";")[0]
            if inasm or not code.strip() or code.strip().startswith("."):
                continue
            assert not re.search(r"\ba\[?\d", code) and "accvgpr" not in code, f"{name}: compiler touched an accumulation register: {line}"
            assert not re.search(r"\bm0\b", code), f"{name}: compiler uses m0: {line}"
            used = [int(g.group(1)) for g in re.finditer(r"\bv(\d+)\b", code)]
            for g in re.finditer(r"\bv\[(\d+):(\d+)\]", code):
                used += [int(g.group(1)), int(g.group(2))]
            for v in used:
                assert v < 64 or v > 251, f"{name}: compiler allocated v{v}, inside the range the asm owns: {line}"
        assert n_asm > 40, f"{name}: inline asm markers missing from the assembly"
        loop = re.search(r"WR_D0_\d+:(.*?)WR_END_\d+:", m.group(2), re.S)
        assert loop and "#ASMEND" not in loop.group(1), f"{name}: the step loop must be a single asm statement"
    metas = re.findall(r"\.name:\s+(_ZN5patch19prefill_kernel_wreg\w*)\n(?:(?!\.name:).)*?\.vgpr_spill_count:\s+(\d+)", text, re.S)
    if not metas:   # older metadata order: spill count first
        metas = [(n, c) for c, n in re.findall(r"\.vgpr_spill_count:\s+(\d+)(?:(?!\.vgpr_spill_count:).)*?\.name:\s+(_ZN5patch19prefill_kernel_wreg\w*)", text, re.S)]
    assert len(metas) == 3, f"kernel metadata not found: {metas}"
    for n, c in metas:
        assert int(c) == 0, f"{n}: {c} vector registers spilled"
    assert len(re.findall(r"\.agpr_count:\s+256", text)) >= 3


@pytest.mark.parametrize("source,kernel,at_least", [("gemm_decode.hip", "decode_kernel", 4), ("gemm_mid.hip", "mid_kernel", 4),
                                                   ("gemm_prefill.hip", "prefill_kernel_lds", 2), ("gemm_prefill.hip", "prefill_kernel_areg", 6), ("quant4.hip", "prefill4_kernel", 8)])
def test_kernels_with_untracked_loads_do_not_spill(source, kernel, at_least):
    """decode_kernel and mid_kernel issue their loads from asm statements and wait for them in a later one; until
    that wait the destinations must stay where the loads write them.  A spill (or any scratch use) of such a register
    would store a value that is still in flight, so every instantiation must report none.  prefill_kernel_lds issues its
    matrix instructions from asm statements: a spill or a scratch copy of an accumulator behind one of them would store
    a value the matrix pipe is still writing (seen once: a duplicated loop body made the register allocator spill
    accumulators, and some outputs came out wrong now and then)."""
    import subprocess
    from paper_2509_23410_amd import build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *[f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")], "-c", "--cuda-device-only",
           "-Rpass-analysis=kernel-resource-usage", "-I", os.path.join(ROOT, "include"), "-I", build.CSRC,
           "-o", os.devnull, os.path.join(build.CSRC, source)]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-2000:]
    blocks = re.split(r"remark: Function Name: ", r.stdout)[1:]
    seen = 0
    for b in blocks:
        name = b.split()[0]
        if kernel not in name:
            continue
        seen += 1
        get = lambda key: int(re.search(re.escape(key) + r":\s*(\d+)", b).group(1))
        assert get("VGPRs Spill") == 0 and get("SGPRs Spill") == 0, f"{name} spills"
        assert get("ScratchSize [bytes/lane]") == 0, f"{name} uses scratch memory"
        assert get("VGPRs") <= 256 and get("AGPRs") == 0, name
    assert seen >= at_least, f"expected several instantiations of {kernel}, saw {seen}"


def test_no_flat_memory_instructions(tmp_path):
    """Every pointer the kernels dereference is device memory.  A pointer that reached a kernel inside a by-value struct
    or through scalar selects loses its address space unless the code restores it; the compiler then emits flat
    instructions (and reads read-only tables with vector loads), which cost the 4-bit decode launch a quarter of its
    time.  The generated assembly of every source must contain none."""
    import subprocess
    from paper_2509_23410_amd import build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    for src in build.sources():
        out = tmp_path / (os.path.basename(src) + ".s")
        cmd = [hipcc, *[f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")], "-S", "--cuda-device-only",
               "-I", os.path.join(ROOT, "include"), "-I", build.CSRC, "-o", str(out), src]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout[-2000:]
        text = out.read_text()
        flat = [l.strip() for l in text.splitlines() if re.match(r"\s+flat_(load|store|atomic)", l)]
        assert not flat, f"{os.path.basename(src)}: {len(flat)} flat instructions, e.g. {flat[0]}"
        if os.path.basename(src) == "quant4.hip":
            # table entries of the 4-bit product kernel come through scalar loads
            body = re.search(r"^_ZN5patch14decode4_kernelILi128ELi1ELi1ENS_5Q4OneE.*?^\.Lfunc_end", text, re.S | re.M)
            assert body and len(re.findall(r"\bs_load_dword\b", body.group(0))) >= 2


@pytest.mark.parametrize("source,pattern,at_least", [
    # prefill_kernel_lds: tile 128 / 64 x whole / split x blocks of 256 / 128 rows; prefill_kernel_areg: (128, 128), (64, 128),
    # (64, 256) x whole / split; prefill4_kernel: tile 128 / 64 x blocks of 128 / 256 rows x whole / split
    ("gemm_prefill.hip", r"_ZN5patch1[89]prefill_kernel_(?:lds|areg)\w+", 14), ("quant4.hip", r"_ZN5patch15prefill4_kernel\w+", 8)])
def test_lds_prefill_kernel_leaves_its_accumulators_alone(tmp_path, source, pattern, at_least):
    """The prefill kernels built on mma_step issue their matrix instructions from asm statements, so the compiler does not
    know that an accumulator is still being written when the statement ends (the hardware does not interlock a read of
    it either).  From the first of those statements to the wait states in front of the output stage no
    compiler-generated instruction may touch an accumulator register: no copy, no spill, no reuse."""
    import subprocess
    from paper_2509_23410_amd import build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = tmp_path / (source + ".s")
    cmd = [hipcc, *[f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")], "-S", "--cuda-device-only",
           "-I", os.path.join(ROOT, "include"), "-I", build.CSRC, "-o", str(out), os.path.join(build.CSRC, source)]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-2000:]
    text = out.read_text()
    bodies = re.findall(r"^(" + pattern + r"):.*?\n(.*?)^\.Lfunc_end", text, re.S | re.M)
    assert len(bodies) >= at_least, [b[0] for b in bodies]

    def regs(tok):
        out_ = set()
        for g in re.finditer(r"\bv\[(\d+):(\d+)\]", tok):
            out_.update(range(int(g.group(1)), int(g.group(2)) + 1))
        for g in re.finditer(r"\bv(\d+)\b", tok):
            out_.add(int(g.group(1)))
        return out_

    for name, body in bodies:
        lines = body.splitlines()
        since, inasm, last = {}, False, None        # accumulator register -> line of the first matrix instruction into it
        for i, line in enumerate(lines):
            if "#ASMSTART" in line:
                inasm = True
            elif "#ASMEND" in line:
                inasm = False
            elif inasm and re.match(r"\s+v_s?mfmac?_", line):
                for r in regs(line.split(",")[0]):
                    since.setdefault(r, i)
                last = i
        # 8 accumulator tiles of 16 registers with blocks of 256 rows, 4 with 128 (the template argument BM)
        bm = re.search(r"prefill_kernel_ldsILi\d+ELb[01]ELi(\d+)E|prefill_kernel_aregILi\d+ELi(\d+)E", name)
        bm = bm or re.search(r"prefill4_kernelILi\d+ELi(\d+)E()", name)
        want = 128 if (bm.group(1) or bm.group(2)) == "256" else 64
        assert len(since) == want and last is not None, (name, len(since))
        # ... and up to the wait states the kernel itself puts before its output stage reads the accumulators.  A tile
        # that no matrix instruction has written yet is still a constant (zero) to the compiler, which may keep other
        # values in its registers until then: only instructions behind the tile's first matrix instruction count.
        end = next(i for i in range(last, len(lines)) if "s_nop 15" in lines[i])
        inasm = False
        for i, line in enumerate(lines[:end]):
            if "#ASMSTART" in line:
                inasm = True
                continue
            if "#ASMEND" in line:
                inasm = False
                continue
            code = line.split(";")[0]
            if inasm or not code.strip() or code.strip().startswith(".") or code.strip().endswith(":"):
                continue
            touched = {r for r in regs(code) if r in since and i > since[r]}
            assert not touched, f"{name}: compiler instruction touches accumulator registers {sorted(touched)[:4]}: {line.strip()}"
