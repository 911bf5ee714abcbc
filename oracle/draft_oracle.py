"""CPU oracle of one layer of draft-tree expansion.

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing in the product path).  Plain numpy, written from what the
paper defines, in its notation; shares no code with the native implementation.

What is written out here (paper, "Tree Expansion Phase"; "Dynamic Expansion Stage", first paragraphs):
  * a node u has the value v(u) = product over its path of P_D(x_w | c_w), the root 1;
  * a selected node u is given K children, the K most probable tokens under P_D(. | c_u);
  * the candidates of the next layer are those children, and the method looks at their values sorted in
    descending order, v_i(1) >= ... >= v_i(N_i) (Eq. 1), to decide how many to keep.

Readings taken where the text is silent:
  E1. Values are carried as scores = log v: a child's score is its parent's score plus log P_D(x | c_u), one
      float32 addition (the draft head's log-probabilities come in as float32).  The order of values and of scores
      is the same; a sum of logs does not underflow at depth 13.
  E2. "K child nodes by sampling from P_D" is read as the K most probable tokens, as the paper's own sentence on the
      initial number of nodes per layer says ("determined by the top-K probability"), and as EAGLE does.
  E3. Ties: among equal log-probabilities the lower token index comes first; among candidates of equal score the one
      of the earlier parent row, then of the lower rank under that parent, comes first.  NaNs must not occur.
  E4. Every comparison is made on the float32 values as they are: nothing here rounds except the one addition of E1.
  * Pins: the paper prints no numeric example of an expansion, so no expected value is taken from it;
    tests/test_draft_oracle_pins.py pins this function by selection written as repeated maximum search, by the
    product definition of v(u), and by the property the Tree Reranking Phase relies on (a child's value never
    exceeds its parent's, so the best m nodes form a subtree).
"""
from __future__ import annotations

import numpy as np


def expand_layer(score, cu_N, logp, K: int):
    """One layer.  Sequence b owns the selected nodes (rows) cu_N[b] .. cu_N[b+1]-1; score[r] is log v of row r
    (float32), logp[r] the draft head's log-probabilities of its next token (float32 [V]).
    Returns per sequence a tuple (cand_score float32 [n_b*K], cand_parent int32 [n_b*K] (row within the sequence),
    cand_token int32 [n_b*K]), the candidates in descending order of score."""
    score = np.asarray(score, dtype=np.float32)
    logp = np.asarray(logp, dtype=np.float32)
    V = logp.shape[1]
    assert 1 <= K <= V
    out = []
    for b in range(len(cu_N) - 1):
        r0, r1 = int(cu_N[b]), int(cu_N[b + 1])
        cs, cp, ct = [], [], []
        for r in range(r0, r1):
            # the K most probable tokens of the row: descending log-probability, lower token first among equals
            order = np.lexsort((np.arange(V), -logp[r].astype(np.float64)))[:K]
            for tok in order:
                cs.append(np.float32(score[r] + logp[r, tok]))     # float32 + float32, rounded once
                cp.append(r - r0)
                ct.append(int(tok))
        cs = np.array(cs, dtype=np.float32)
        # descending score; equal scores in the order they were generated (parent row, then rank)
        order = np.lexsort((np.arange(len(cs)), -cs.astype(np.float64)))
        out.append((cs[order], np.array(cp, np.int32)[order], np.array(ct, np.int32)[order]))
    return out
