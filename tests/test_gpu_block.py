"""GPU parity of one decoder block against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import synth
from tests.parity import assert_appended_rows, assert_block_close, errors

pytestmark = pytest.mark.gpu


def _device_run(shape, w, K, V, x, S, cap, mode, grid, threads, repeats, taps):
    from paper_2604_23553_amd.harness import DeviceStack
    ds = DeviceStack(shape, cap, 1, 1)
    try:
        ds.set_options(mode=mode, grid=grid, threads=threads)
        ds.load_layer(0, w)
        ds.load_kv(0, K, V, S)
        ds.set_inputs(x, S)
        outs = []
        for _ in range(repeats):
            ds.block_decode(0)
            ds.check()
            outs.append(ds.result().copy())
        k_all, v_all = ds.export_kv(0, 0, 0, cap)
        tap = None
        if taps:
            tap = {n: ds.tap(i, shape.ffn if n == "m" else shape.hidden)
                   for i, n in enumerate(("q", "m", "g", "attn"))}
    finally:
        ds.close()
    return outs, (k_all, v_all), tap


def run_block(orc, shape, seed, S, cap, mode=0, grid=None, threads=None, taps=False, repeats=1):
    """The block on the product library; with taps=True once more on the profiling
    build of the same sources (the only one with the test taps), whose output must
    be the product's bit for bit."""
    import paper_2604_23553_amd as cf
    w = synth.layer_weights(shape, seed, 0)
    K, V = synth.kv_cache(shape, seed, 0, S, cap)
    x = synth.x_input(shape, seed)
    print(f"[case] shape={shape.name or shape.hidden} seed={seed} S={S} cap={cap} mode={mode} grid={grid} threads={threads}", flush=True)
    outs, kv_dev, _ = _device_run(shape, w, K, V, x, S, cap, mode, grid, threads, repeats, False)
    tap = None
    if taps:
        with cf.profile_build():
            outs_p, kv_p, tap = _device_run(shape, w, K, V, x, S, cap, mode, grid, threads, 1, True)
        assert np.array_equal(outs_p[0].view(np.uint16), outs[0].view(np.uint16)), "profiling build differs from the product"
        assert np.array_equal(kv_p[0].view(np.uint16), kv_dev[0].view(np.uint16))
    Ko, Vo = K[0].copy(), V[0].copy()
    ref, otaps = orc.block_decode(shape, w, Ko, Vo, S, orc.half_to_real(x[0]), taps=True)
    return outs, kv_dev, (Ko, Vo), orc.real_to_half(ref), tap, otaps, (w, orc.half_to_real(x[0]))


def check_block(orc, shape, seed, S, cap, **kw):
    outs, (kg, vg), (Ko, Vo), ref16, tap, otaps, (w, x_real) = run_block(orc, shape, seed, S, cap, **kw)
    ma, rl = assert_block_close(outs[0][0], ref16, "block output")
    # appended rows: correct roundings of the oracle's unrounded values within the fp32 evaluation
    # bound; every other slot untouched (bit-exact, NaN poison included)
    assert_appended_rows(kg[:, S], vg[:, S], shape, w, x_real, otaps, "block")
    assert np.array_equal(np.ascontiguousarray(kg[:, :S]).view(np.uint16), np.ascontiguousarray(Ko[:, :S]).view(np.uint16))
    assert np.array_equal(np.ascontiguousarray(vg[:, :S]).view(np.uint16), np.ascontiguousarray(Vo[:, :S]).view(np.uint16))
    assert np.isnan(kg[:, S + 1:].astype(np.float32)).all() and np.isnan(vg[:, S + 1:].astype(np.float32)).all()
    for o in outs[1:]:
        assert np.array_equal(o.view(np.uint16), outs[0].view(np.uint16)), "not bit-identical run to run"
    if tap is not None:
        # (the whole-stack kernel keeps the down projection in registers and passes the
        # attention output on as tagged words: no workspace copy of either)
        names = ("q", "m") if kw.get("mode") == 2 else ("q", "m", "g", "attn")
        for n in names:
            e = errors(tap[n], otaps[n])
            assert e[0] < 2e-3 and e[1] < 2e-4, f"intermediate {n}: {e}"
    return ma, rl


@pytest.mark.parametrize("mode", [0, 1, 2, -1])
def test_small_block_config(orc, mode):
    """hidden 512, 8 heads x 64, rotary 16, FFN 2048, 128 cached positions."""
    check_block(orc, synth.SMALL_BLOCK, synth.MASTER_SEED, 128, 129, mode=mode, taps=True, repeats=3)


@pytest.mark.parametrize("S", [0, 1, 31, 32, 33, 63, 64, 65, 257, 1000])
def test_context_lengths_and_ragged_rows(orc, S):
    check_block(orc, synth.SMALL_BLOCK, 7 + S, S, S + 3, mode=0, taps=True)


@pytest.mark.parametrize("grid,threads", [(1, 256), (7, 512), (64, 256), (256, 256), (300, 512), (1024, 512)])
def test_launch_shapes(orc, grid, threads):
    check_block(orc, synth.SMALL_BLOCK, 11, 200, 201, mode=0, grid=grid, threads=threads, taps=True)


@pytest.mark.parametrize("mode", [0, 1, 2, -1])
def test_pythia_2_8b_block(orc, mode):
    """hidden 2560, 32 heads x 80, rotary 20, FFN 10240, 1024 cached positions."""
    check_block(orc, synth.PYTHIA_2_8B, synth.MASTER_SEED, 1024, 1025, mode=mode, taps=True, repeats=3)


@pytest.mark.parametrize("mode", [0, 2])
def test_pythia_6_9b_block(orc, mode):
    check_block(orc, synth.PYTHIA_6_9B, synth.MASTER_SEED, 333, 334, mode=mode, taps=True, repeats=2)


@pytest.mark.parametrize("shape", [
    synth.ModelShape(576, 9, 64, 16, 1160, name="ragged-h576"),     # K not a multiple of 512
    synth.ModelShape(640, 8, 80, 20, 2048, name="d80-h640"),
    synth.ModelShape(1024, 8, 128, 32, 520, name="d128-f520"),
    synth.ModelShape(512, 8, 64, 0, 2048, name="no-rotary"),
    synth.ModelShape(512, 8, 64, 64, 2048, name="full-rotary"),
])
def test_odd_shapes(orc, shape):
    check_block(orc, shape, 5, 70, 80, mode=0, taps=True)
    check_block(orc, shape, 5, 70, 71, mode=1, grid=40, threads=256)


def test_last_slot_of_the_cache(orc):
    check_block(orc, synth.SMALL_BLOCK, 3, 95, 96, mode=0)


def test_packed_row_constants():
    """Behind the tensors a packed layer carries, per row of the QKV and MLP-up
    matrices, s = W gamma and c = W beta + b of the LayerNorm in front of them
    (the whole-stack kernel completes the LayerNorm with them in the epilogue).
    They are checked here against the plain products in float64; the QKV rows
    are in the packed order the header documents (per head q | k | v, rotary
    pair (j, j + r/2) adjacent)."""
    from paper_2604_23553_amd.harness import DeviceStack
    shape = synth.ModelShape(640, 8, 80, 20, 2048, name="d80-h640")
    h, f, d, r = shape.hidden, shape.ffn, shape.head_dim, shape.rotary_dims
    w = synth.layer_weights(shape, 11, 0)
    print("[case] packed row constants", flush=True)
    ds = DeviceStack(shape, 16, 1, 1)
    try:
        ds.load_layer(0, w)
        blob = ds.packed[0].cpu().numpy()
    finally:
        ds.close()
    up256 = lambda n: (n + 255) // 256 * 256
    off_up = blob.size - up256(8 * f)
    off_qkv = off_up - up256(8 * 3 * h)
    rc_qkv = blob[off_qkv:off_qkv + 8 * 3 * h].view(np.float32).reshape(3 * h, 2)
    rc_up = blob[off_up:off_up + 8 * f].view(np.float32).reshape(f, 2)
    f64 = lambda a: a.astype(np.float64)
    rows = np.empty(3 * h, dtype=np.int64)
    for p in range(3 * h):
        n, rem = divmod(p, 3 * d)
        c, i = divmod(rem, d)
        dim = ((i >> 1) + (r >> 1 if i & 1 else 0)) if (c < 2 and i < r) else i
        rows[p] = (3 * n + c) * d + dim
    Wq = f64(w["w_qkv"])[rows]
    want_q = np.stack([Wq @ f64(w["ln1_g"]), Wq @ f64(w["ln1_b"]) + f64(w["b_qkv"])[rows]], axis=1)
    Wu = f64(w["w_up"])
    want_u = np.stack([Wu @ f64(w["ln2_g"]), Wu @ f64(w["ln2_b"]) + f64(w["b_up"])], axis=1)
    assert np.allclose(rc_qkv, want_q, rtol=1e-6, atol=1e-7)
    assert np.allclose(rc_up, want_u, rtol=1e-6, atol=1e-7)
