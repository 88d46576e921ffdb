"""Teacher-forced forward of the pipelined decoder (Section 3.3, Eq. 5-6, Fig. 3b): the training
target is fed whole, every token at its grid coordinate, in ONE pass under the boolean matrix of
Fig. 3b, and the loss sums -log P of every next token.  Test infrastructure only; fp64 numpy;
quadratic in the number of tokens.

Eq. 5: the i-th target subsequence becomes [<bos>, Y_i, <eos>]; one empty subsequence [<bos>, <eos>]
is appended so that the model learns to stop opening new ones.
Eq. 6: L = - sum over (i, t) of log P(Yhat_i^{t+1} | Yhat_{<=i}^{<=t}; input): one term for every
token of a subsequence that has a successor; the conditioning set is every token of subsequences
<= i at times <= t, and the whole input.
Reading where the paper is silent: the closing <eos> of a subsequence has no loss term of its own
(nothing follows it) but it belongs to the conditioning set of the later tokens of subsequences
>= i from its own time on, exactly as Algorithm 1 feeds a finished subsequence's last token once.
So every token of the target is a row and a key; the last token of each subsequence is a key only.

The encoder-decoder form (teacher_forced_encdec) is the same pass through oracle/encdec.py's dense
decoder: the matrix of Fig. 3b over the target's tokens, the Manhattan distance of Section 4.3 between
every visible pair, the encoder states of Eq. 1 behind the second attention.

Parity status: pinned in tests/test_oracle_training.py by Fig. 3b's worked example (the target and
its 8 loss terms), by Algorithm 1 run with the target's tokens forced (the incremental decoder of
oracle/pipelined.py gives the same distributions step by step), by an independent PyTorch library
model with its library cross-entropy under a mask enumerated in the test (any schedule; one
subsequence = ordinary language-model loss), and by planted mistakes; the encoder-decoder form by
Algorithm 1 with the target forced through the incremental encoder-decoder decoder and by the
independent PyTorch encoder-decoder of tests/torch_encdec.py with the library's cross-entropy.
"""

import numpy as np

from . import encdec, matrix_form

F = np.float64


def training_target(Y, bos_id, eos_id):
    """Eq. 5: [[bos, Y_1, eos], ..., [bos, Y_n, eos], [bos, eos]]."""
    return [[bos_id] + [int(t) for t in y] + [eos_id] for y in Y] + [[bos_id, eos_id]]


def teacher_forced(model, ctx_tokens, target, delta_t):
    """target: the subsequences of Eq. 5 (lists of token ids).  Returns (logits, nll, loss):
    logits [N, V] for all N tokens of the target in subsequence-major order (row of token j of
    subsequence i: sum of the lengths before i, plus j), nll [N] = -log P(next token) with 0 for
    the last token of each subsequence, loss = sum of nll (Eq. 6)."""
    ctx = np.asarray(ctx_tokens)
    L = ctx.shape[0]
    coords = matrix_form.coordinates(target, delta_t)            # (i, tau, token), subsequence-major
    tokens = np.concatenate([ctx, np.array([c[2] for c in coords], dtype=np.int64)])
    positions = np.concatenate([np.arange(L), np.array([L + (tau - 1) + (i - 1) for i, tau, _ in coords],
                                                       dtype=np.int64)])
    logits = matrix_form.dense_forward(model, tokens, positions, matrix_form.attention_matrix(L, coords))[L:]
    nll = np.zeros(len(coords), dtype=F)
    r = 0
    for sub in target:
        for j in range(len(sub)):
            if j + 1 < len(sub):
                row = logits[r]
                m = row.max()
                nll[r] = m + np.log(np.exp(row - m).sum()) - row[sub[j + 1]]
            r += 1
    return logits, nll, float(nll.sum())


def _nll(logits, target):
    nll = np.zeros(logits.shape[0], dtype=F)
    r = 0
    for sub in target:
        for j in range(len(sub)):
            if j + 1 < len(sub):
                row = logits[r]
                m = row.max()
                nll[r] = m + np.log(np.exp(row - m).sum()) - row[sub[j + 1]]
            r += 1
    return nll


def teacher_forced_encdec(model, ctx_tokens, target, delta_t):
    """The same for an oracle.encdec.EncDecModel: returns (logits [N, V], nll [N], loss)."""
    coords = matrix_form.coordinates(target, delta_t)
    ii = np.array([c[0] for c in coords])
    tt = np.array([c[1] for c in coords])
    mask = (ii[None, :] <= ii[:, None]) & (tt[None, :] <= tt[:, None])
    distance = np.abs(tt[:, None] - tt[None, :]) + np.abs(ii[:, None] - ii[None, :])
    logits = encdec.dense_decoder_forward(model, model.encode(ctx_tokens), [c[2] for c in coords], mask, distance)
    nll = _nll(logits, target)
    return logits, nll, float(nll.sum())
