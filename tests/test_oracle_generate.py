"""Pins of the oracle's greedy generation loop (the steps either side of the
decode stack: embedding lookup before it, final LayerNorm + LM head + argmax
after it; paper Sec. 2.3 replays the graph once per generated token; the rule
that picks a token is not named in the paper, the largest logit is taken).
CPU only."""
import numpy as np

import synth


def _setup(seed=7, L=2, S=4, steps=5, vocab=97):
    sh = synth.ModelShape(64, 4, 16, 4, 256, n_layers=L)
    layers = synth.stack_weights(sh, seed)
    cap = S + steps + 1
    kv = [synth.kv_cache(sh, seed, l, S, cap) for l in range(L)]
    Ks, Vs = [k[0][0].copy() for k in kv], [k[1][0].copy() for k in kv]
    head = synth.lm_head(sh, seed, vocab=vocab)
    embed = synth.embedding(sh, seed, vocab=vocab)
    tokens = list(np.random.default_rng(seed).integers(0, vocab, S + 1))
    return sh, layers, Ks, Vs, head, embed, tokens, S


def test_branches_switched_off_reduce_to_a_closed_form(orc):
    """With W_dense = W_down = 0 and zero biases every block returns its input,
    so token[t+1] = argmax(W_lm LN(embed[token[t]])) - evaluated here with plain
    numpy in float64 (textbook LayerNorm, library matmul)."""
    sh, layers, Ks, Vs, head, embed, tokens, S = _setup()
    for w in layers:
        for n in ("w_dense", "b_dense", "w_down", "b_down"):
            w[n] = np.zeros_like(w[n])
    got = orc.generate(sh, layers, Ks, Vs, head, embed, tokens, S, 5)
    assert got[:S + 1] == tokens and len(got) == S + 6
    g, b, W = (head[n].astype(np.float64) for n in ("lnf_g", "lnf_b", "w_lm"))
    t = tokens[S]
    for step in range(5):
        x = embed[t].astype(np.float64)
        z = (x - x.mean()) / np.sqrt(x.var() + sh.ln_eps) * g + b
        t = int(np.argmax(W @ z))
        assert got[S + 1 + step] == t


def test_loop_is_the_composition_of_single_steps_and_appends_one_row_per_step(orc):
    sh, layers, Ks, Vs, head, embed, tokens, S = _setup(seed=11)
    K0 = [k.copy() for k in Ks]
    Ks1, Vs1 = [k.copy() for k in Ks], [v.copy() for v in Vs]
    trace = []
    got = orc.generate(sh, layers, Ks, Vs, head, embed, tokens, S, 4, trace=trace)
    # by hand, one step at a time
    cur, pos = list(tokens), S
    for step in range(4):
        h16, _ = orc.stack_decode(sh, layers, Ks1, Vs1, pos, np.ascontiguousarray(embed[cur[pos]]))
        lg = orc.lm_head_logits(sh, head, orc.half_to_real(h16))
        assert np.array_equal(h16, trace[step][0]) and np.array_equal(lg, trace[step][1])
        cur.append(int(np.argmax(lg)))
        pos += 1
    assert cur == got
    for l in range(sh.n_layers):
        assert np.array_equal(Ks[l].view(np.uint16), Ks1[l].view(np.uint16))
        changed = np.any(Ks[l].view(np.uint16) != K0[l].view(np.uint16), axis=(0, 2))
        assert list(np.nonzero(changed)[0]) == [S, S + 1, S + 2, S + 3]     # rows S.. of every head, nothing else


def test_next_token_takes_the_lowest_index_among_equal_maxima(orc):
    sh = synth.ModelShape(64, 4, 16, 4, 256)
    head = synth.lm_head(sh, 5, vocab=50)
    hidden = synth.x_input(sh, 5)[0]
    tok, lg = orc.next_token(sh, head, hidden)
    assert tok == int(np.argmax(lg)) and lg[tok] == lg.max()
    head["w_lm"][40] = head["w_lm"][tok]
    head["w_lm"][3] = head["w_lm"][tok]
    tok2, lg2 = orc.next_token(sh, head, hidden)
    assert lg2[3] == lg2[40] == lg2[tok] and tok2 == min(3, tok)
