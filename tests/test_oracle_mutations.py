"""The pins must have teeth: each plausible mistake below is planted into a
COPY of the oracle's source (on the CPU, in a temp dir), and at least one pin
has to fail against that build."""
import os
import subprocess

import pytest

from oracle import ds_oracle as orc
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(orc.__file__), "ds_oracle.c")

MUTATIONS = [
    ("outer index uses the wrong stride", "pos += k[j] * d->strides[j];", "pos += k[j] * d->strides[nd - 2 - j];"),
    ("outer term dropped", "pos += k[j] * d->strides[j];", "pos += 0;"),
    ("inner stride ignored", "row_t + es * c * inner_stride", "row_t + es * c"),
    ("rank advances by one row too few", "r += inner;", "r += inner - 1;"),
    ("odometer runs first index fastest", "int j = (int)nd - 2;\n    while (j >= 0) {\n      if (++k[j] < d->shape[j]) break;\n      k[j] = 0;\n      --j;\n    }\n    if (j < 0) break;",
     "int j = 0;\n    while (j <= (int)nd - 2) {\n      if (++k[j] < d->shape[j]) break;\n      k[j] = 0;\n      ++j;\n    }\n    if (j > (int)nd - 2) break;"),
    ("padding not zeroed", "memset(image, 0, (size_t)total);\n  for (size_t i = 0; i < n; ++i) copy_shard(&d[i], image, 1);", "for (size_t i = 0; i < n; ++i) copy_shard(&d[i], image, 1);"),
    ("offsets not aligned", "at = round_up(at + (uint64_t)b, align);", "at = at + (uint64_t)b;"),
    ("image tail not rounded", "*total = at;", "*total = n ? d[n - 1].file_offset + (uint64_t)dso_shard_bytes(&d[n - 1]) : 0;"),
    ("bf16 taken as 4 bytes", "case DSO_BF16: return 2;", "case DSO_BF16: return 4;"),
    ("unpack writes the image instead", "else memcpy(row_t, row_i, (size_t)(es * inner));", "else memcpy(row_i, row_t, (size_t)(es * inner));"),
    ("scalar shard skipped", "if (to_image) memcpy(img, base, (size_t)es); else memcpy(base, img, (size_t)es);", ";"),
]

PIN_CALLS = [
    pins.test_itemsizes,
    pins.test_layout_hand_fixture,
    lambda: pins.test_layout_closed_form_and_invariants(256),
    pins.test_image_hand_fixture,
    pins.test_contiguous_shards_are_numpy_tobytes,
    lambda: [pins.test_strided_views_index_encoding(dt) for dt in ("u8", "bf16", "f32", "i64")],
    pins.test_brute_force_tiny_inputs,
    pins.test_pack_overwrites_stale_image_bytes,
    lambda: pins.test_unpack_roundtrip_and_sentinel(lambda: pins.W.fragmentation(100, max_bytes=1 << 12, seed=33)),
]


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(what, old, new, tmp_path, monkeypatch):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation anchor not unique: {what}"
    mutated = tmp_path / "ds_oracle_mut.c"
    mutated.write_text(text.replace(old, new))
    so = tmp_path / "libmut.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-pthread", "-o", str(so), str(mutated)], check=True)
    monkeypatch.setattr(orc, "_lib", orc.bind(str(so)))
    caught = False
    for call in PIN_CALLS:
        try:
            call()
        except (AssertionError, ValueError):
            caught = True
            break
    assert caught, f"no pin noticed: {what}"


# ---- the oracles written in Python: the same game on their source text ------------------------------------
import importlib.util
import sys
import types

import test_ckpt_format as fpins
from oracle import ckpt_format as fmt_mod
from oracle import image_compress as ic_mod

PY_MUTATIONS = [
    # (what, module, old, new)
    ("files: offsets not rounded up to the alignment", fmt_mod, "at[f] += size + (-size % align)", "at[f] += size"),
    ("files: one running offset for all files", fmt_mod, "offs.append(at[f])\n        at[f] += size + (-size % align)",
     "offs.append(at[0])\n        at[0] += size + (-size % align)"),
    ("files: regions start where the file before STARTS", fmt_mod, "begins.append(run)\n        run += at[f]",
     "begins.append(run)\n        run += at[f - 1] if f else 0"),
    ("files: a file gets the table's entries of the NEXT file", fmt_mod, "[t for t, g in zip(tensors, file_of) if g == f], appends[f])",
     "[t for t, g in zip(tensors, file_of) if g == (f + 1) % n_files], appends[f])"),
    ("file: chunks of the log not padded to 8 bytes", fmt_mod, 'out += b"\\0" * (-len(data) % 8)', "pass"),
    ("file: chunk index in arrival order, not sorted", fmt_mod, "for c in sorted(chunks):", "for c in chunks:"),
    ("file: sequence numbers shared by all objects", fmt_mod, "seq = seen.get(object_id, 0)\n        seen[object_id] = seq + 1",
     "seq = seen.get(0, 0)\n        seen[0] = seq + 1"),
    ("file: footer without the tensor count", fmt_mod, "align, T, E, len(tensors), len(chunks),", "align, T, E, 0, len(chunks),"),
    ("compress: a block is constant if it equals its first BYTE", ic_mod, "keep[k] = 0 if np.all(units == units[0]) else 1",
     "keep[k] = 0 if np.all(units == units[0][0]) else 1"),
    ("compress: positions count all blocks", ic_mod, "pos[k + 1] = pos[k] + keep[k]", "pos[k + 1] = pos[k] + 1"),
    ("compress: the pattern is the block's last unit", ic_mod, "patterns[k] = units[0]", "patterns[k] = units[-1]"),
    ("decompress: kept blocks read from their own block number", ic_mod, "at = int(pos[k]) * block_bytes", "at = k * block_bytes"),
]


def _mutated(module, old, new):
    path = module.__file__
    text = open(path).read()
    assert text.count(old) == 1, f"mutation anchor not unique: {old!r}"
    m = types.ModuleType(module.__name__ + "_mut")
    m.__file__ = path
    exec(compile(text.replace(old, new), path, "exec"), m.__dict__)
    return m


@pytest.mark.parametrize("what,module,old,new", PY_MUTATIONS, ids=[m[0] for m in PY_MUTATIONS])
def test_planted_mistake_in_a_python_oracle_is_caught(what, module, old, new, monkeypatch):
    mut = _mutated(module, old, new)
    if module is fmt_mod:
        monkeypatch.setattr(fpins, "fmt", mut)
        calls = [fpins.test_oracle_builds_the_hand_written_file, fpins.test_oracle_rules_on_random_files,
                 fpins.test_rank_files_by_hand_and_against_the_single_file_layout]
        errors = (AssertionError, ValueError, fmt_mod.FormatError, mut.FormatError, IndexError, KeyError)
    else:
        monkeypatch.setitem(sys.modules, "oracle.image_compress", mut)
        import oracle
        monkeypatch.setattr(oracle, "image_compress", mut, raising=False)
        calls = [pins.test_image_compress_block_elision_by_hand_and_by_brute_force]
        errors = (AssertionError, ValueError, IndexError)
    caught = False
    for call in calls:
        try:
            call()
        except errors:
            caught = True
            break
    assert caught, f"no pin noticed: {what}"
