"""Host-only checks of the C-ABI library (no GPU): it loads, exports every symbol
the header declares, and its layout / byte arithmetic is right."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import synth
import paper_2604_23553_amd as cf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="cfpp.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cfpp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 20
    L = cf.lib()
    for n in names:
        assert hasattr(L, n), f"{n} is declared in cfpp.h but not exported"


def test_product_library_has_no_profiling_entry_points():
    """Tracer switches, test taps and calibration kernels live in the profiling
    build only (include/cfpp_profile.h); that build exports them beside the ABI."""
    extra = sorted(set(declared_functions("cfpp_profile.h")) - set(declared_functions()))
    assert "cfpp_debug_read" in extra and "cfpp_stream_copy" in extra
    L = cf.lib()
    for n in extra:
        assert not hasattr(L, n), f"{n} is exported by the product library"
    with cf.profile_build() as P:
        for n in extra + declared_functions():
            assert hasattr(P, n), f"{n} is missing from the profiling library"
        assert cf.lib() is P
    assert cf.lib() is L
    text = open(os.path.join(ROOT, "include", "cfpp.h")).read()
    assert "PROFILE_SKIP" not in text and "debug_read" not in text


def test_binding_has_the_same_names():
    for n in declared_functions():
        if n in ("cfpp_status_string", "cfpp_last_error"):
            continue
        assert hasattr(cf, n), f"binding lacks {n}"


@pytest.mark.parametrize("shape,max_seq,weights,kv_read", [
    (synth.SMALL_BLOCK, 129, 6_304_768, 262_144),
    (synth.PYTHIA_2_8B, 1025, 157_352_960, 10_485_760),
    (synth.PYTHIA_6_9B, 2049, 402_759_680, 33_554_432),
])
def test_sizes_and_algorithmic_bytes(shape, max_seq, weights, kv_read):
    cfg = cf.Config.from_shape(shape, max_seq)
    assert cf.cfpp_validate_config(cfg) == 0
    h, f = shape.hidden, shape.ffn
    assert (12 * h * h + 13 * h) * 2 == weights
    # every section of the packed blob is 256-byte aligned; for these shapes no padding is needed.
    # Behind the tensors: two fp32 constants per row of the QKV and MLP-up matrices, derived at packing
    assert cf.cfpp_packed_layer_bytes(cfg) == weights + (3 * h + f) * 8
    assert cf.cfpp_kv_layer_bytes(cfg) == 2 * h * max_seq * 2
    S = max_seq - 1
    got = cf.cfpp_algorithmic_bytes(cfg, [S], 1)
    assert got == weights + kv_read + 2 * h * 2 + 2 * h * 2
    assert cf.cfpp_workspace_bytes(cfg) > 0


def test_stack_bytes_match_the_stated_target_workload():
    # 32 x (157,352,960 + 41,943,040 + 10,240) + x/out = 6,377.8 MB
    cfg = cf.Config.from_shape(synth.PYTHIA_2_8B, 4097)
    b = cf.cfpp_algorithmic_bytes(cfg, [4096], 32)
    assert b == 32 * (157_352_960 + 41_943_040 + 10_240) + 2 * 2560 * 2
    assert abs(b / 1e6 - 6377.8) < 0.05


def test_batch_bytes_count_each_sequence():
    cfg = cf.Config.from_shape(synth.PYTHIA_6_9B, 8193, max_batch=8)
    lens = synth.seq_lens(synth.MASTER_SEED, 8, 1024, 8192)
    b = cf.cfpp_algorithmic_bytes(cfg, lens.tolist(), 1)
    assert b == 402_759_680 + 16_384 * int(lens.sum()) + 8 * 16_384 + 8 * 4096 * 4


@pytest.mark.parametrize("kw,status", [
    (dict(hidden=513), -1),                      # hidden != heads * head_dim
    (dict(rotary_dims=17), -1),                  # odd rotary width
    (dict(rotary_dims=66), -1),                  # wider than the head
    (dict(flags=4), -1),                         # unknown flag bit
    (dict(max_seq=0), -1),
    (dict(n_heads=4, head_dim=96, hidden=384), -2),   # head_dim without a kernel
    (dict(ffn=2052), -2),                        # not a multiple of 8
    (dict(n_layers=65), -2),
    (dict(max_batch=65), -2),
])
def test_validate_config_rejects(kw, status):
    base = dict(hidden=512, n_heads=8, head_dim=64, rotary_dims=16, ffn=2048, n_layers=1, max_seq=16,
                max_batch=1, rope_base=10000.0, ln_eps=1e-5, flags=0)
    base.update(kw)
    cfg = cf.Config(**base)
    assert cf.cfpp_validate_config(cfg) == status
    assert cf.lib().cfpp_last_error() != b""
    assert cf.cfpp_packed_layer_bytes(cfg) == 0 and cf.cfpp_workspace_bytes(cfg) == 0


def test_argument_errors_without_a_gpu():
    cfg = cf.Config.from_shape(synth.SMALL_BLOCK, 16)
    L = cf.lib()
    assert L.cfpp_validate_config(None) == -1
    with pytest.raises(cf.CfppError) as e:
        cf.cfpp_algorithmic_bytes(cfg, [16], 1)          # pos == max_seq
    assert e.value.status == -1
    with pytest.raises(cf.CfppError):
        cf.cfpp_pack_layer(cfg, {n: 0 for n in cf.binding.LAYER_TENSORS}, 0)   # null pointers
    with pytest.raises(cf.CfppError):
        cf.cfpp_create(cfg, 0, 1 << 20)                  # null workspace
    with pytest.raises(cf.CfppError):
        cf.cfpp_create(cfg, 4096 + 8, 1 << 20)           # misaligned workspace
    with pytest.raises(cf.CfppError) as e:
        cf.cfpp_create(cfg, 4096, 16)                    # too small
    assert e.value.status == -3
    assert L.cfpp_stack_replay(None, None) == -1
    assert L.cfpp_block_decode(None, None, None, None, None, 1, None, None) == -1
    assert L.cfpp_block_decode_static(None, None, None, None, None, 1, None, None) == -1
    # the built-in workspace of the allocation-free entry point has a stated maximum
    big = cf.Config.from_shape(synth.PYTHIA_6_9B, 1 << 20, max_batch=8)
    assert cf.cfpp_workspace_bytes(big) > (16 << 20)
    with pytest.raises(cf.CfppError) as e:
        cf.cfpp_block_decode_static(big, 4096, 4096, 4096, 4096, 1, 8192)
    assert e.value.status == -3
    assert b"ok" == L.cfpp_status_string(0)


def test_qkv_packing_permutation_is_a_bijection_that_pairs_rotary_rows():
    # mirror of the row order the header documents: within q and k of a head,
    # packed rows (2j, 2j+1) hold canonical dims (j, j + r/2)
    for d, r in ((64, 16), (80, 20), (128, 32), (64, 0), (64, 64)):
        H = 3
        def canon(p):
            n, rem = divmod(p, 3 * d)
            c, i = divmod(rem, d)
            if c < 2 and i < r:
                i = (i >> 1) + (r >> 1) if (i & 1) else (i >> 1)
            return (3 * n + c) * d + i
        rows = [canon(p) for p in range(3 * H * d)]
        assert sorted(rows) == list(range(3 * H * d))
        for n in range(H):
            for c in (0, 1):
                for j in range(r // 2):
                    p = (3 * n + c) * d + 2 * j
                    assert rows[p] == (3 * n + c) * d + j and rows[p + 1] == (3 * n + c) * d + j + r // 2
