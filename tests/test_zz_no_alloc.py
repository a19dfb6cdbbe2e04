"""The allocation-free entry point (cfpp_block_decode_static: the workspace is a
fixed array in the library's device image) against cfpp_block_decode with a
caller-owned workspace, through the C ABI: two calls in a row, the second with a
smaller input; then a batch of sequences, and the stated size limit."""
import numpy as np
import pytest

import synth
from tests.parity import assert_appended_rows, assert_block_close, ulp16

pytestmark = pytest.mark.gpu


def both_ways(shape, seed, lens, cap):
    """One block step through the context entry point (launch mode 0) and through the
    static one, each on its own copy of the cache.  Returns (out, appended K, V) twice."""
    import torch
    import paper_2604_23553_amd as cf
    from paper_2604_23553_amd.harness import DeviceStack
    lens = np.atleast_1d(np.asarray(lens, dtype=np.int32))
    B = len(lens)
    w = synth.layer_weights(shape, seed, 0)
    K, V = synth.kv_cache(shape, seed, 0, lens, cap, B)
    x = synth.x_input(shape, seed, B)
    res = []
    for static in (False, True):
        ds = DeviceStack(shape, cap, B, 1)
        try:
            ds.load_layer(0, w)
            ds.load_kv(0, K, V, lens)
            ds.set_inputs(x, lens)
            if static:
                cf.cfpp_block_decode_static(ds.cfg, ds.packed[0], ds.kv[0], ds.x, ds.pos, B, ds.out, ds.s)
                ds.stream.synchronize()
            else:
                ds.set_options(mode=0)
                ds.block_decode(0)
                ds.check()
            out = ds.result().copy()
            rows = [ds.export_kv(0, b, int(lens[b]), 1) for b in range(B)]
            untouched = ds.export_kv(0, 0, 0, int(lens[0]))
        finally:
            ds.close()
        res.append((out, rows, untouched))
    return res, (w, K, V, x, lens)


def check_case(orc, shape, seed, lens, cap):
    (ctx_way, static_way), (w, K, V, x, lens) = both_ways(shape, seed, lens, cap)
    print(f"[case] static entry point {shape.name} lens={list(lens)}", flush=True)
    for b in range(len(lens)):
        # against the existing entry point: the same kernels on another workspace; the rotary
        # table is built on the device here and on the host there (both in double)
        assert_block_close(static_way[0][b], ctx_way[0][b], f"static vs context, sequence {b}")
        for a, c in zip(static_way[1][b], ctx_way[1][b]):
            a64, c64 = a[:, 0].astype(np.float64), c[:, 0].astype(np.float64)
            assert (np.abs(a64 - c64) <= ulp16(c64)).all(), f"appended row, sequence {b}: more than one fp16 step apart"
        # and against the oracle
        ref, taps = orc.block_decode(shape, w, K[b].copy(), V[b].copy(), int(lens[b]), orc.half_to_real(x[b]), taps=True)
        assert_block_close(static_way[0][b], orc.real_to_half(ref), f"static vs oracle, sequence {b}")
        assert_appended_rows(static_way[1][b][0][:, 0], static_way[1][b][1][:, 0], shape, w, orc.half_to_real(x[b]), taps,
                             f"static, sequence {b}")
    same = all(np.array_equal(static_way[0][b].view(np.uint16), ctx_way[0][b].view(np.uint16)) for b in range(len(lens)))
    print(f"[result] static entry point bit-identical to the context one: {same}", flush=True)
    for a, c in zip(static_way[2], ctx_way[2]):
        assert np.array_equal(a.view(np.uint16), c.view(np.uint16)), "cached rows were touched"


def test_two_calls_in_a_row_the_second_smaller(orc):
    big = synth.ModelShape(2560, 32, 80, 20, 10240, n_layers=1, name="pythia-2.8b-block")
    check_case(orc, big, 71, [300], 301)
    check_case(orc, synth.SMALL_BLOCK, 72, [70], 75)           # smaller shape, shorter cache: the array is re-armed
    check_case(orc, synth.SMALL_BLOCK, 73, [5], 75)            # same configuration again: no set-up kernel this time


def test_batch_of_sequences(orc):
    check_case(orc, synth.SMALL_BLOCK, 74, [3, 64, 17], 80)


def test_sizes_beyond_the_built_in_array_are_refused():
    import paper_2604_23553_amd as cf
    from paper_2604_23553_amd.harness import DeviceStack
    ds = DeviceStack(synth.SMALL_BLOCK, 16, 1, 1)
    try:
        big = cf.Config.from_shape(synth.PYTHIA_6_9B, 1 << 20, max_batch=8)
        assert cf.cfpp_workspace_bytes(big) > (16 << 20)
        with pytest.raises(cf.CfppError) as e:
            cf.cfpp_block_decode_static(big, ds.packed[0], ds.kv[0], ds.x, ds.pos, 1, ds.out, ds.s)
        assert e.value.status == -3 and "16777216" in str(e.value)
    finally:
        ds.close()
