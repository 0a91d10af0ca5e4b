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
