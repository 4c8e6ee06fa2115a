"""The device image of the built library must export the static workspace array of
gx_layer_bwd_static: the HIP runtime looks the array up by name when the entry point asks for its
device address, and a symbol that is local to its code object cannot be found (the lookup then
ends the process).  Checked on the file itself, no GPU needed: the device code objects are cut out
of the library's fat binary and their symbol tables read."""
import os
import struct

import pytest

from paper_2504_03662_amd import binding as gx

MAGIC = b"__CLANG_OFFLOAD_BUNDLE__"


def _code_objects(blob):
    """(triple, bytes) of every entry of every offload bundle found in `blob`."""
    out, pos = [], 0
    while True:
        pos = blob.find(MAGIC, pos)
        if pos < 0:
            return out
        n, = struct.unpack_from("<Q", blob, pos + len(MAGIC))
        cur = pos + len(MAGIC) + 8
        for _ in range(n):
            off, size, tlen = struct.unpack_from("<QQQ", blob, cur)
            triple = blob[cur + 24:cur + 24 + tlen].decode()
            out.append((triple, blob[pos + off:pos + off + size]))
            cur += 24 + tlen
        pos += len(MAGIC)


def _symbols(elf):
    """(name, binding, size) of every entry of an ELF64 object's .symtab / .dynsym."""
    assert elf[:4] == b"\x7fELF" and elf[4] == 2
    shoff, = struct.unpack_from("<Q", elf, 0x28)
    shentsize, shnum = struct.unpack_from("<HH", elf, 0x3A)
    secs = [struct.unpack_from("<IIQQQQIIQQ", elf, shoff + i * shentsize) for i in range(shnum)]
    syms = []
    for (_, stype, _, _, off, size, link, _, _, entsize) in secs:
        if stype not in (2, 11):            # SHT_SYMTAB, SHT_DYNSYM
            continue
        stroff = secs[link][4]
        for k in range(size // entsize):
            name, info, _, _, _, ssize = struct.unpack_from("<IBBHQQ", elf, off + k * entsize)
            end = elf.index(b"\0", stroff + name)
            syms.append((elf[stroff + name:end].decode(), info >> 4, ssize, stype))
    return syms


def test_static_scratch_is_an_exported_device_symbol():
    if not os.path.exists(gx.LIB_PATH):
        from paper_2504_03662_amd.build import build
        build(verbose=False)
    blob = open(gx.LIB_PATH, "rb").read()
    objs = [(t, b) for t, b in _code_objects(blob) if "gfx950" in t and b[:4] == b"\x7fELF"]
    assert objs, "no gfx950 code object in the library"
    found = []
    for _, elf in objs:
        found += [s for s in _symbols(elf) if s[0].endswith("scratch") and s[2] == 64 << 20]
    assert found, "the 64 MiB scratch array is not in any device code object"
    # STB_GLOBAL = 1; it must also sit in the dynamic symbol table (type 11), which is what the loader reads
    assert all(binding == 1 for _, binding, _, _ in found), found
    assert any(stype == 11 for _, _, _, stype in found), found
