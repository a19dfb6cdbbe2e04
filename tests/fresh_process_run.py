"""One decode step of a small stack on the GPU, printed as a digest of the fp16
output and the appended K/V rows: run as `python -m tests.fresh_process_run MODE`
by the determinism test, which compares the digest of a fresh process with its
own."""
import hashlib
import sys

import numpy as np

import synth

SHAPE = synth.ModelShape(512, 8, 64, 16, 2048, n_layers=4, name="neox-h512-x4")
SEED, S, CAP = 77, 133, 140


def digest(mode: int, replays: int = 1) -> str:
    from paper_2604_23553_amd.harness import DeviceStack
    ds = DeviceStack(SHAPE, CAP, 1, SHAPE.n_layers)
    try:
        for l in range(SHAPE.n_layers):
            ds.load_layer(l, synth.layer_weights(SHAPE, SEED, l))
            K, V = synth.kv_cache(SHAPE, SEED, l, S, CAP)
            ds.load_kv(l, K, V, S)
        ds.set_options(mode=mode)
        ds.set_inputs(synth.x_input(SHAPE, SEED), S)
        ds.capture()
        h = None
        for _ in range(replays):
            ds.replay()
            ds.check()
            m = hashlib.sha256()
            m.update(np.ascontiguousarray(ds.result()).view(np.uint8).tobytes())
            for l in range(SHAPE.n_layers):
                k, v = ds.export_kv(l, 0, S, 1)
                m.update(np.ascontiguousarray(k).view(np.uint8).tobytes())
                m.update(np.ascontiguousarray(v).view(np.uint8).tobytes())
            if h is not None and m.hexdigest() != h:
                raise AssertionError("replays of one process differ")
            h = m.hexdigest()
        return h
    finally:
        ds.close()


if __name__ == "__main__":
    print("digest", digest(int(sys.argv[1])), flush=True)
