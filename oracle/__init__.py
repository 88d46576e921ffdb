"""CPU oracle for the pipelined decoder (Section 3 of the paper: Eq. 2-4,
Algorithm 1, the dependency rule of Section 3.2 and the attention pattern of
Fig. 3b).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 numpy statement
of what the method computes.  It exists to check the HIP library; it is never
part of the product path.  Only the test-suite, the smoke check and the
benchmark's cpu_baseline leg may import it.  It shares no code with the HIP
path and does not import it.

Modules
  primitives.py   layer norm / RMS norm / GELU / SiLU / rotary embedding / linear maps
  model.py        weights in fp64 + the causal pass over the context (Eq. 1 analogue)
  controller.py   Algorithm 1 as a loop around an arbitrary "decoder" callable
  pipelined.py    formulation F1: incremental per-query loop with explicit visible sets
  matrix_form.py  formulation F2: full recompute of the flattened sequence under the
                  boolean attention matrix of Fig. 3b
  splitk.py       log-sum-exp merge of softmax partials (exact identity used by the GPU)
  encdec.py       the encoder-decoder form the paper itself runs (Eq. 1 encoder states, cross-attention,
                  bucketed relative-position bias on the Manhattan distance of Section 4.3)
  training.py     the teacher-forced forward of Section 3.3: the training target of Eq. 5 fed whole under
                  the matrix of Fig. 3b, and the loss of Eq. 6

Parity status: the logit VALUES on random weights are printed nowhere in the
paper; they are pinned by (a) an independent dense transformer written with
PyTorch library ops in the tests (S=1 == ordinary greedy decoding; no-overlap
schedule == plain causal decoding; arbitrary schedules == the brute-force
enumerated mask), (b) F1 == F2, (c) the paper's worked example of Fig. 2 with
a scripted decoder, and (d) closed forms of the schedule.
"""
