"""Greedy generation through the C ABI (embedding -> stack -> final LayerNorm +
LM head -> next token, position advanced on the device) against the oracle's
loop.  The oracle follows the GPU's own tokens (teacher forcing), so one
near-tie cannot derail the comparison of everything behind it."""
import numpy as np
import pytest

import synth
from tests.parity import assert_block_close

pytestmark = pytest.mark.gpu

SHAPE = synth.ModelShape(512, 8, 64, 16, 2048, n_layers=4, name="neox-h512-x4")
VOCAB = 1000        # not a multiple of the grid: ragged last workgroup


def _world(seed, S, steps):
    cap = S + steps + 1
    layers = synth.stack_weights(SHAPE, seed)
    kv = [synth.kv_cache(SHAPE, seed, l, S, cap) for l in range(SHAPE.n_layers)]
    head = synth.lm_head(SHAPE, seed, vocab=VOCAB)
    embed = synth.embedding(SHAPE, seed, vocab=VOCAB)
    tokens = [int(t) for t in np.random.default_rng(seed).integers(0, VOCAB, S + 1)]
    return cap, layers, kv, head, embed, tokens


def _device(cap, layers, kv, head, embed, S, mode):
    from paper_2604_23553_amd.harness import DeviceStack
    ds = DeviceStack(SHAPE, cap, 1)
    for l in range(SHAPE.n_layers):
        ds.load_layer(l, layers[l])
        ds.load_kv(l, kv[l][0], kv[l][1], S)
    ds.load_lm(head, embed)
    ds.set_options(mode=mode)
    return ds


def _follow(orc, layers, kv, head, embed, tokens_gpu, S, steps):
    """The oracle fed with the GPU's tokens: per step its hidden state, logits and K/V."""
    Ks = [k[0][0].copy() for k in kv]
    Vs = [k[1][0].copy() for k in kv]
    out = []
    for i in range(steps):
        pos = S + i
        x = np.ascontiguousarray(embed[tokens_gpu[pos]])
        h16, _ = orc.stack_decode(SHAPE, layers, Ks, Vs, pos, x)
        tok, lg = orc.next_token(SHAPE, head, h16)
        out.append((h16, lg, tok))
    return out, Ks, Vs


@pytest.mark.parametrize("mode", [0, 2])
def test_generation_graph_matches_oracle_over_64_steps(orc, mode):
    S, steps = 37, 64
    print(f"[case] generation mode={mode} S={S} steps={steps}", flush=True)
    cap, layers, kv, head, embed, tokens = _world(23553, S, steps)
    ds = _device(cap, layers, kv, head, embed, S, mode)
    try:
        ds.set_tokens(tokens, S)
        ds.generate_capture()
        hidden = []
        for _ in range(steps):
            ds.replay()
            ds.stream.synchronize()
            hidden.append(ds.out[0].cpu().numpy().copy())      # the stack's output of this step
        ds.check()
        got = ds.tokens.cpu().numpy()
        assert int(ds.pos[0].item()) == S + steps
        assert list(got[: S + 1]) == tokens and np.all(got[S + steps + 1:] == 0)
        ref, Ks, Vs = _follow(orc, layers, kv, head, embed, got, S, steps)
        # Greedy choice per step: where the oracle's two best logits are further apart than ten
        # times the logit error of this step (oracle's LM head on the GPU's hidden state against
        # the oracle's own logits), the token must be the oracle's; in a near-tie both leaders are
        # correct greedy choices and the GPU's must be one of them.  (The oracle follows the GPU's
        # tokens, so a near-tie does not derail the comparison of the later steps.)
        exact, ties = 0, []
        for i, (h16, lg, tok) in enumerate(ref):
            g = int(got[S + 1 + i])
            assert 0 <= g < VOCAB
            assert_block_close(hidden[i], h16, f"hidden state of step {i}")
            err = float(np.abs(orc.lm_head_logits(SHAPE, head, orc.half_to_real(hidden[i])) - lg).max())
            top = np.argsort(lg)[-2:]
            margin = float(lg[top[1]] - lg[top[0]])
            if margin > 10 * err:
                assert g == tok, f"step {i}: token {g}, oracle {tok} (margin {margin:.3e}, logit error {err:.3e})"
            else:
                ties.append((i, margin, err))
                assert g in top, f"step {i}: token {g} is neither leader of a near-tie"
            exact += g == tok
        print(f"[result] mode {mode}: {exact}/{steps} tokens identical to the oracle's choice; near-ties {ties}", flush=True)
        assert len(ties) <= 2
        # the K/V rows appended on the way are the oracle's (fp16: equal up to one rounding step)
        for l in range(SHAPE.n_layers):
            k, v = ds.export_kv(l, 0, S, steps)
            for a, b in ((k, Ks[l][:, S:S + steps]), (v, Vs[l][:, S:S + steps])):
                a, b = a.astype(np.float64), b.astype(np.float64)
                assert np.abs(a - b).max() <= 2e-2 and np.linalg.norm(a - b) <= 5e-3 * np.linalg.norm(b)
    finally:
        ds.close()


def test_prompt_through_the_gemm_kernels_then_generation(orc):
    """The whole flow from an empty cache: the prompt's embedding rows through the prompt-sized
    kernels (cfpp_stack_prefill_gemm), then the generation graph from the prompt's last token on;
    the oracle does the same with its token-by-token prompt loop and follows the GPU's tokens."""
    S, steps, seed = 45, 24, 4711
    cap = S + steps + 1
    print(f"[case] prompt of {S} tokens, then {steps} generated", flush=True)
    layers = synth.stack_weights(SHAPE, seed)
    kv = [synth.kv_cache(SHAPE, seed, l, 0, cap) for l in range(SHAPE.n_layers)]
    head = synth.lm_head(SHAPE, seed, vocab=VOCAB)
    embed = synth.embedding(SHAPE, seed, vocab=VOCAB)
    tokens = [int(t) for t in np.random.default_rng(seed).integers(0, VOCAB, S + 1)]
    ds = _device(cap, layers, kv, head, embed, 0, 2)
    try:
        X = np.ascontiguousarray(embed[tokens[:S]])        # the tokens at positions 0 .. S-1
        got_prompt = ds.prefill_gemm(X, 0, 0, 128)
        ds.check()
        ds.set_tokens(tokens, S)                           # the loop starts with token S at position S
        ds.generate_capture()
        hidden = []
        for _ in range(steps):
            ds.replay()
            ds.stream.synchronize()
            hidden.append(ds.out[0].cpu().numpy().copy())
        ds.check()
        got = ds.tokens.cpu().numpy()
        assert int(ds.pos[0].item()) == S + steps and list(got[: S + 1]) == tokens
        Ks = [k[0][0].copy() for k in kv]
        Vs = [k[1][0].copy() for k in kv]
        want_prompt, _ = orc.prefill(SHAPE, layers, Ks, Vs, 0, X)
        for t in range(S):
            assert_block_close(got_prompt[t], want_prompt[t], f"prompt token {t}")
        ties = 0
        for i in range(steps):
            pos = S + i
            h16, _ = orc.stack_decode(SHAPE, layers, Ks, Vs, pos, np.ascontiguousarray(embed[got[pos]]))
            tok, lg = orc.next_token(SHAPE, head, h16)
            assert_block_close(hidden[i], h16, f"hidden state of step {i}")
            err = float(np.abs(orc.lm_head_logits(SHAPE, head, orc.half_to_real(hidden[i])) - lg).max())
            top = np.argsort(lg)[-2:]
            g = int(got[pos + 1])
            if float(lg[top[1]] - lg[top[0]]) > 10 * err:
                assert g == tok, f"step {i}: token {g}, oracle {tok}"
            else:
                ties += 1
                assert g in top, f"step {i}: token {g} is neither leader of a near-tie"
        assert ties <= 2
    finally:
        ds.close()


def test_single_steps_logits_and_bit_identical_rerun(orc):
    S, steps = 20, 6
    print(f"[case] generation call by call S={S} steps={steps}", flush=True)
    cap, layers, kv, head, embed, tokens = _world(7, S, steps)
    runs = []
    for rep in range(2):
        ds = _device(cap, layers, kv, head, embed, S, 2)
        try:
            ds.set_tokens(tokens, S)
            hid, lgs = [], []
            for _ in range(steps):
                ds.generate_step(want_logits=True)
                ds.check()
                hid.append(ds.out[0].cpu().numpy().copy())
                lgs.append(ds.logits.cpu().numpy().copy())
            runs.append((ds.tokens.cpu().numpy().copy(), hid, lgs))
        finally:
            ds.close()
    assert np.array_equal(runs[0][0], runs[1][0])
    for a, b in zip(runs[0][1] + runs[0][2], runs[1][1] + runs[1][2]):
        assert np.array_equal(a.view(np.uint32) if a.dtype == np.float32 else a.view(np.uint16),
                              b.view(np.uint32) if b.dtype == np.float32 else b.view(np.uint16))
    got, hid, lgs = runs[0]
    ref, _, _ = _follow(orc, layers, kv, head, embed, got, S, steps)
    for i, (h16, lg, tok) in enumerate(ref):
        assert_block_close(hid[i], h16, f"hidden state of step {i}")
        # logits of the GPU's own hidden state: LayerNorm + 512-term dot products in fp32
        lg_own = orc.lm_head_logits(SHAPE, head, orc.half_to_real(hid[i]))
        assert np.abs(lgs[i].astype(np.float64) - lg_own).max() <= 1e-4
        assert int(got[S + 1 + i]) == int(np.argmax(lgs[i]))          # lowest index of the GPU's own maximum


def test_bad_token_and_end_of_cache_raise_the_flag(orc):
    from paper_2604_23553_amd import CfppError
    S, steps = 8, 2
    cap, layers, kv, head, embed, tokens = _world(3, S, steps)
    ds = _device(cap, layers, kv, head, embed, S, 2)
    try:
        bad = list(tokens)
        bad[S] = VOCAB + 5
        ds.set_tokens(bad, S)
        ds.generate_step()
        with pytest.raises(CfppError):
            ds.check()
        ds.set_tokens(tokens, S)
        for _ in range(steps + 1):                # cap = S + steps + 1 rows: positions S .. S + steps fit
            ds.generate_step()
        ds.check()
        assert int(ds.pos[0].item()) == cap
        ds.generate_step()                        # position == max_seq: nothing runs, flag raised
        with pytest.raises(CfppError):
            ds.check()
        assert int(ds.pos[0].item()) == cap
    finally:
        ds.close()


@pytest.mark.parametrize("vocab", [1, 7, 100, 4096])
def test_lm_head_with_fewer_rows_than_workgroups_and_ties(orc, vocab):
    """Vocabularies smaller than the grid (workgroups without rows), a single
    row, and duplicated rows (equal logits: the lowest index wins)."""
    import paper_2604_23553_amd as cf
    from paper_2604_23553_amd.harness import DeviceStack
    print(f"[case] LM head vocab={vocab}", flush=True)
    head = synth.lm_head(SHAPE, 9, vocab=vocab)
    if vocab >= 7:
        head["w_lm"][vocab - 1] = head["w_lm"][2]          # two equal logits
        head["w_lm"][5] = head["w_lm"][2]
    hidden = synth.x_input(SHAPE, 9)
    ds = DeviceStack(SHAPE, 8, 1, 1)
    try:
        ds.load_lm(head, synth.embedding(SHAPE, 9, vocab=vocab))
        ds.set_tokens([0, 0], 1)
        import torch
        ds.out[:1].copy_(torch.from_numpy(hidden))
        cf.cfpp_lm_next(ds.ctx, ds.lm, ds.out, ds.tokens, ds.pos, ds.logits, ds.s)
        ds.check()
        lg = ds.logits.cpu().numpy()
        want = orc.lm_head_logits(SHAPE, head, orc.half_to_real(hidden[0]))
        assert np.abs(lg.astype(np.float64) - want).max() <= 1e-4
        if vocab >= 7:
            assert lg[2] == lg[5] == lg[vocab - 1]
        assert int(ds.tokens[2].item()) == int(np.argmax(lg))      # numpy: first of equal maxima
        if vocab >= 7:
            # make the tied rows the winners: the pick must be row 2
            z = orc.layernorm(orc.half_to_real(hidden[0]), head["lnf_g"], head["lnf_b"], SHAPE.ln_eps)
            row = (z / np.abs(z).max()).astype(np.float16)          # aligned with the normalised vector: largest logit
            head["w_lm"][[2, 5, vocab - 1]] = row * np.float16(4.0)
            ds.load_lm(head, synth.embedding(SHAPE, 9, vocab=vocab))
            ds.set_tokens([0, 0], 1)
            cf.cfpp_lm_next(ds.ctx, ds.lm, ds.out, ds.tokens, ds.pos, ds.logits, ds.s)
            ds.check()
            lg = ds.logits.cpu().numpy()
            assert lg[2] == lg.max() and lg[5] == lg[2] == lg[vocab - 1]
            assert int(ds.tokens[2].item()) == 2
    finally:
        ds.close()
