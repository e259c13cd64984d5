"""The C-ABI library loads without a GPU and exports every symbol the headers under include/ declare."""
import glob
import os
import re

import numpy as np
import pytest

import paper_1610_02496_amd as pk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for path in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        text = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)
        names.update(re.findall(r"\b(saber_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 15
    lib = pk.load_library()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(pk.EXPORTS) == names


def test_struct_layouts_match_header():
    import ctypes
    assert ctypes.sizeof(pk.Options) == 16 * 4
    assert ctypes.sizeof(pk.Stats) == 23 * 8
    o = pk.options_default()
    assert (o.n_chunks, o.block_threads, o.tile_tokens, o.stage_phi, o.profile) == (0, 0, 0, 1, 0)


def header_struct_fields(name):
    text = open(os.path.join(ROOT, "include", "saber.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    body = re.search(r"typedef struct %s \{(.*?)\} %s;" % (name, name), text, flags=re.S).group(1)
    fields = []
    for decl in body.split(";"):
        m = re.match(r"\s*(int32_t|int64_t|double|float|uint32_t|uint64_t)\s+(\w+)(\[(\d+)\])?\s*$", decl)
        if m:
            fields.append((m.group(2), m.group(1), int(m.group(4)) if m.group(4) else 0))
    return fields


def test_binding_structs_mirror_the_header_field_by_field():
    import ctypes
    ctype_of = {"int32_t": ctypes.c_int32, "int64_t": ctypes.c_int64, "double": ctypes.c_double, "float": ctypes.c_float,
                "uint32_t": ctypes.c_uint32, "uint64_t": ctypes.c_uint64}
    for cname, cls in (("saber_options", pk.Options), ("saber_stats", pk.Stats)):
        want = header_struct_fields(cname)
        assert len(want) >= 10
        got = [(n, t) for n, t in cls._fields_]
        assert [n for n, _ in got] == [n for n, _, _ in want], cname
        for (n, t), (_, ct, cnt) in zip(got, want):
            assert t == (ctype_of[ct] * cnt if cnt else ctype_of[ct]), (cname, n)


def test_validation_happens_before_any_device_work():
    """Bad arguments are rejected on the host, GPU or not."""
    dp = np.array([0, 2], dtype=np.int64)
    with pytest.raises(pk.SaberError) as e:
        pk.Saber(dp, np.array([0, 7], dtype=np.int32), 2, 3, 0.1, 0.01, 1)
    assert e.value.code == pk.binding.SABER_EINVAL and "word id" in str(e.value)
    with pytest.raises(pk.SaberError) as e:
        pk.Saber(np.array([0, 2, 1], dtype=np.int64), np.array([0, 1], dtype=np.int32), 2, 3, 0.1, 0.01, 1)
    assert e.value.code == pk.binding.SABER_EINVAL
    with pytest.raises(pk.SaberError) as e:
        pk.Saber(dp, np.array([0, 1], dtype=np.int32), 2, 1 << 20, 0.1, 0.01, 1)
    assert e.value.code == pk.binding.SABER_ERANGE
    # K = 262144 needs 18 topic bits, which leaves 14 bits for a count: a document of 2^14 tokens is refused
    with pytest.raises(pk.SaberError) as e:
        pk.Saber(np.array([0, 1 << 14], dtype=np.int64), np.zeros(1 << 14, dtype=np.int32), 2, 262144, 0.1, 0.01, 1)
    assert e.value.code == pk.binding.SABER_ERANGE and "count bits" in str(e.value)


def test_no_gpu_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(pk.SaberError) as e:
        pk.Saber(np.array([0, 2], dtype=np.int64), np.array([0, 1], dtype=np.int32), 2, 3, 0.1, 0.01, 1)
    assert e.value.code == pk.binding.SABER_EDEVICE
