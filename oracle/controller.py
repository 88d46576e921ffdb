"""Algorithm 1 (decoding loop) around an arbitrary decoder callable.
Test infrastructure only.

Reading of the paper used here
  * Loop iteration t (1-based) first opens a new subsequence when (t-1) mod dt == 0
    and fewer than sub_max exist, so k = min(sub_max, ceil(t/dt)) (Eq. 2), then asks
    the decoder for one new token per existing subsequence (Eq. 3) and appends it
    to every subsequence that has not finished.
  * A subsequence has finished once it received <eos>, or (an addition of this
    build, not in the paper) once it holds `sub_tokens` generated tokens.
  * The loop stops as soon as every subsequence opened SO FAR has finished, or
    after time_max iterations.
  * The result drops <bos> and the closing <eos>.

The loop takes the steps of Algorithm 1 in the paper's order (open, decode, append, test for
termination): the plain definition of a control loop is that loop, so this is by necessity the
same sequence of steps as the paper's pseudo-code, written out from the description in Section 3.2.
"""


def pipelined_decode(decoder, delta_t, time_max, sub_max, bos_id, eos_id=-1, sub_tokens=None):
    """Run Algorithm 1.

    decoder(G, t) -> sequence of len(G) token ids: the next token of every
    subsequence in G (entries for finished subsequences are ignored).  G is the
    list of subsequences, each a list of token ids starting with bos_id.

    Returns (result, steps, emitted) where result is G without <bos>/<eos>,
    steps the number of iterations run, and emitted[t-1] a dict
    {subsequence index (1-based): token appended in iteration t}.
    """
    assert delta_t >= 1 and time_max >= 0 and sub_max >= 0
    G, done, by_eos = [], [], []
    k = 0
    emitted = []
    steps = 0
    for t in range(1, time_max + 1):
        if (t - 1) % delta_t == 0 and k < sub_max:
            G.append([bos_id])
            done.append(False)
            by_eos.append(False)
            k += 1
        if k == 0:
            break
        new = decoder(G, t)
        out = {}
        for i in range(k):
            if not done[i]:
                tok = int(new[i])
                G[i].append(tok)
                out[i + 1] = tok
                if eos_id >= 0 and tok == eos_id:
                    done[i] = by_eos[i] = True
                elif sub_tokens is not None and len(G[i]) - 1 >= sub_tokens:
                    done[i] = True
        emitted.append(out)
        steps = t
        if all(done[:k]):
            break
    result = [g[1:-1] if e else g[1:] for g, e in zip(G, by_eos)]
    return result, steps, emitted
