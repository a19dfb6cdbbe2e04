"""GPU parity of prompt processing (cfpp_stack_prefill) against the CPU oracle,
through the C ABI: every token's output, the rows appended to every layer's
cache, and a decode step that continues behind the prompt."""
import numpy as np
import pytest

import synth
from tests.parity import assert_appended_rows, assert_block_close, errors

pytestmark = pytest.mark.gpu

TINY_STACK = synth.ModelShape(512, 8, 64, 16, 2048, n_layers=4, name="neox-h512-x4")


def _build(shape, seed, pos0, cap, max_batch):
    from paper_2604_23553_amd.harness import DeviceStack
    L = shape.n_layers
    ds = DeviceStack(shape, cap, max_batch, L)
    ws = [synth.layer_weights(shape, seed, l) for l in range(L)]
    kvs = [synth.kv_cache(shape, seed, l, pos0, cap, max_batch) for l in range(L)]
    for l in range(L):
        ds.load_layer(l, ws[l])
        ds.load_kv(l, kvs[l][0], kvs[l][1], pos0)
    return ds, ws, kvs


def _check_prompt(orc, shape, seed, pos0, T, max_batch, b=0, then_decode=True, gemm_rows=0, row_check_every=1):
    cap = pos0 + T + 2
    print(f"[case] prefill shape={shape.name} seed={seed} pos0={pos0} T={T} max_batch={max_batch} b={b} gemm_rows={gemm_rows}", flush=True)
    ds, ws, kvs = _build(shape, seed, pos0, cap, max_batch)
    try:
        ds.set_options(mode=0)
        X = synth.x_input(shape, seed + 1, batch=T)
        got = ds.prefill_gemm(X, pos0, b, gemm_rows) if gemm_rows else ds.prefill(X, pos0, b)
        ds.check()
        Ks = [kv[0][b].copy() for kv in kvs]
        Vs = [kv[1][b].copy() for kv in kvs]
        want16, _ = orc.prefill(shape, ws, Ks, Vs, pos0, X)
        for t in range(T):
            assert_block_close(got[t], want16[t], f"token {t}")
        # rows appended to every layer's cache of sequence b; nothing else of the cache touched
        for l in range(shape.n_layers):
            kg, vg = ds.export_kv(l, b, 0, cap)
            if l == 0:
                # the first layer reads each token's own input row, the same bits on both sides: its
                # rows must be correct roundings of the oracle's unrounded values
                for t in range(0, T, row_check_every):
                    _, taps = orc.block_decode(shape, ws[0], kvs[0][0][b].copy(), kvs[0][1][b].copy(), pos0 + t,
                                               orc.half_to_real(X[t]), taps=True)
                    assert_appended_rows(kg[:, pos0 + t], vg[:, pos0 + t], shape, ws[0], orc.half_to_real(X[t]), taps,
                                         f"token {t} layer 0")
            else:   # deeper layers see an input that already carries the earlier layers' rounding
                for g_, w_ in ((kg, Ks[l]), (vg, Vs[l])):
                    e = errors(g_[:, pos0:pos0 + T], w_[:, pos0:pos0 + T])
                    assert e[0] <= 2e-2 and e[1] <= 5e-3, f"appended rows, layer {l}: {e}"
            assert np.array_equal(np.ascontiguousarray(kg[:, :pos0]).view(np.uint16),
                                  np.ascontiguousarray(kvs[l][0][b][:, :pos0]).view(np.uint16))
            assert np.isnan(kg[:, pos0 + T:].astype(np.float32)).all() and np.isnan(vg[:, pos0 + T:].astype(np.float32)).all()
            for other in range(max_batch):
                if other != b:
                    ko, _ = ds.export_kv(l, other, 0, cap)
                    assert np.isnan(ko[:, pos0:].astype(np.float32)).all(), "another sequence's cache was written"
        if then_decode and b == 0:
            # one decode step behind the prompt reads what the prompt left in the caches
            x1 = synth.x_input(shape, seed + 2)
            ds.set_inputs(x1, pos0 + T)
            ds.stack_decode()
            ds.check()
            ref16, _ = orc.stack_decode(shape, ws, Ks, Vs, pos0 + T, x1[0])
            assert_block_close(ds.result()[0], ref16, "decode step behind the prompt")
    finally:
        ds.close()


@pytest.mark.parametrize("pos0,T,max_batch,b", [
    (5, 19, 8, 0),        # groups of 8, 8 and 3 behind five cached positions
    (0, 7, 3, 0),         # groups of 3, 3 and 1 from an empty cache
    (3, 9, 8, 2),         # into the cache of the third sequence
    (0, 1, 8, 0),         # a single token
])
def test_prompt_through_the_tiny_stack(orc, pos0, T, max_batch, b):
    _check_prompt(orc, TINY_STACK, 17, pos0, T, max_batch, b)


def test_prompt_at_the_2_8b_shape(orc):
    shape = synth.ModelShape(2560, 32, 80, 20, 10240, n_layers=2, name="pythia-2.8b-x2")
    _check_prompt(orc, shape, 23, 100, 11, 8)


# The same prompts through the prompt-sized kernels (cfpp_stack_prefill_gemm): LayerNorm launch,
# four GEMMs on the matrix cores and one causal-attention launch per layer and pass.
@pytest.mark.parametrize("pos0,T,max_batch,b,rows", [
    (5, 19, 8, 0, 128),       # one pass, most of its tile padding
    (0, 7, 3, 0, 128),        # from an empty cache
    (3, 9, 8, 2, 256),        # into the cache of the third sequence
    (0, 1, 8, 0, 128),        # a single token
    (2, 150, 2, 1, 128),      # two passes (128 + 22): the second attends over the first one's rows
    (0, 200, 1, 0, 256),      # several key tiles and query blocks, ragged at both ends
])
def test_prompt_through_the_tiny_stack_with_the_gemm_kernels(orc, pos0, T, max_batch, b, rows):
    _check_prompt(orc, TINY_STACK, 19, pos0, T, max_batch, b, gemm_rows=rows)


def test_prompt_at_the_2_8b_shape_with_the_gemm_kernels(orc):
    shape = synth.ModelShape(2560, 32, 80, 20, 10240, n_layers=2, name="pythia-2.8b-x2")
    _check_prompt(orc, shape, 29, 60, 70, 1, gemm_rows=128)


def test_gemm_prompt_with_head_dim_128_and_tanh_gelu(orc):
    # the third head size of the attention launch (two dimensions per lane), with the other GELU reading
    shape = synth.ModelShape(1024, 8, 128, 32, 4096, n_layers=2, flags=synth.FLAG_TANH_GELU, name="neox-h1024-d128-x2")
    _check_prompt(orc, shape, 31, 7, 90, 1, gemm_rows=128)


# The cases above are small enough that every product splits K (few tiles) and the parts meet in
# k_pf_reduce.  These two are long enough for the other ways through the GEMM: products that are
# not split and finish out of LDS, with 64-token tiles (600 tokens: QKV and up) and with 128-token
# tiles (2200 tokens: QKV and up; dense and down unsplit with 64-token tiles), at a head size that
# does not divide the 128-column tile (heads cut by tile edges) and a rotated part that is not a
# multiple of 8 dimensions.  Layer-0 rows are held to the rounding bound for every 7th token.


def test_gemm_prompt_long_enough_for_unsplit_products(orc):
    shape = synth.ModelShape(1280, 16, 80, 20, 5120, n_layers=1, name="neox-h1280-x1")
    _check_prompt(orc, shape, 37, 9, 600, 1, gemm_rows=640, row_check_every=7)


def test_gemm_prompt_long_enough_for_128_token_tiles(orc):
    shape = synth.ModelShape(1280, 16, 80, 20, 5120, n_layers=2, name="neox-h1280-x2")
    _check_prompt(orc, shape, 41, 0, 2200, 1, gemm_rows=2304, row_check_every=7)


# From 1024 tokens in a pass the attention launch is the 64-query kernel (16 queries per wavefront,
# every wavefront over all keys of a tile); the 2200-token case above runs it at head size 80,
# these two at 64 and 128, with a pass that ends inside a query block and inside a key tile.
def test_gemm_prompt_wide_attention_head_dim_64(orc):
    shape = synth.ModelShape(512, 8, 64, 16, 2048, n_layers=2, name="neox-h512-x2")
    _check_prompt(orc, shape, 43, 3, 1100, 1, gemm_rows=1152, row_check_every=7)


def test_gemm_prompt_wide_attention_head_dim_128(orc):
    shape = synth.ModelShape(1024, 8, 128, 32, 4096, n_layers=1, flags=synth.FLAG_TANH_GELU, name="neox-h1024-d128-x1")
    _check_prompt(orc, shape, 47, 0, 1030, 1, gemm_rows=1152, row_check_every=7)


def test_gemm_prompt_refuses_the_sequential_form():
    import dataclasses
    from paper_2604_23553_amd import CfppError
    shape = dataclasses.replace(TINY_STACK, flags=synth.FLAG_SEQUENTIAL_RESIDUAL)
    ds, ws, kvs = _build(shape, 1, 0, 12, 1)
    try:
        with pytest.raises(CfppError) as e:
            ds.prefill_gemm(synth.x_input(shape, 2, batch=4), 0, rows=128)
        assert e.value.status == -2
    finally:
        ds.close()


def test_gemm_prompt_requests_that_are_refused():
    import torch
    from paper_2604_23553_amd import CfppError, binding as B
    ds, ws, kvs = _build(TINY_STACK, 1, 0, 12, 8)
    try:
        X = synth.x_input(TINY_STACK, 2, batch=4)
        assert B.cfpp_prefill_scratch_bytes(ds.cfg, 100) == 0 and B.cfpp_prefill_scratch_bytes(ds.cfg, 8192) == 0
        with pytest.raises(CfppError) as e:
            ds.prefill_gemm(X, 9, rows=128)               # positions 9..12 of a cache of 12
        assert e.value.status == -1
        need = B.cfpp_prefill_scratch_bytes(ds.cfg, 128)
        xd = torch.from_numpy(X).to(ds.dev)
        od = torch.zeros_like(xd)
        small = torch.empty(need - 256, dtype=torch.uint8, device=ds.dev)
        with pytest.raises(CfppError) as e:
            B.cfpp_stack_prefill_gemm(ds.ctx, ds.packed, ds.kv, xd, 0, 4, 0, od, small, need - 256, 128, ds.s)
        assert e.value.status == -3                       # scratch too small
        with pytest.raises(CfppError) as e:
            B.cfpp_stack_prefill_gemm(ds.ctx, ds.packed, ds.kv, xd, 0, 4, 0, od, small, need, 100, ds.s)
        assert e.value.status == -1                       # rows not a multiple of 128
        ds.prefill_gemm(X, 8, rows=128)                   # the last four rows fit
        ds.check()
    finally:
        ds.close()


def test_prompt_requests_that_are_refused():
    from paper_2604_23553_amd import CfppError
    ds, ws, kvs = _build(TINY_STACK, 1, 0, 12, 8)
    try:
        X = synth.x_input(TINY_STACK, 2, batch=4)
        ds.set_options(mode=2)
        with pytest.raises(CfppError) as e:
            ds.prefill(X, 0)
        assert e.value.status == -2                       # launch mode 0 only
        ds.set_options(mode=0)
        with pytest.raises(CfppError) as e:
            ds.prefill(X, 9)                              # positions 9..12 of a cache of 12
        assert e.value.status == -1
        with pytest.raises(CfppError) as e:
            ds.prefill(X, 0, b=8)                         # no such sequence
        assert e.value.status == -1
        ds.prefill(X, 8)                                  # the last four rows fit
        ds.check()
    finally:
        ds.close()
