"""Pins of the oracle's logit harvest (unigram successor tables; App. C "adjacency table" tier 1 and
"logit harvesting", Sec. 4 stage 2): a case worked by hand, a library top-k, and invariants."""
import json
import os

import numpy as np
import torch

from oracle import goose_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "harvest_case.json")


def test_hand_worked_case():
    case = json.load(open(GOLDEN))
    w = np.array(case["weights"], dtype=np.float64)
    logits = np.log(w) + np.array([[0.7], [-3.0], [11.0]])      # a shift per row must not matter
    ids, scores = orc.harvest_topk(logits, case["tokens"], case["K"])
    for tok, row in case["expected_rows"].items():
        assert ids[int(tok)].tolist() == row["ids"]
        np.testing.assert_allclose(scores[int(tok)], row["scores"], rtol=1e-12)
    for t in case["untouched_rows"]:
        assert (ids[t] == -1).all() and (scores[t] == 0).all()


def test_against_library_topk_and_invariants():
    rng = np.random.default_rng(3)
    B, V, K = 9, 257, 10
    logits = rng.normal(size=(B, V)) * 3
    tokens = rng.permutation(V)[:B]                               # distinct tokens: every row lands
    ids, scores = orc.harvest_topk(logits, tokens, K)
    tv, ti = torch.topk(torch.from_numpy(logits), K, dim=-1)       # continuous values: no ties
    prob = torch.softmax(torch.from_numpy(logits), dim=-1)
    for i, t in enumerate(tokens):
        assert ids[t].tolist() == ti[i].tolist()
        np.testing.assert_allclose(scores[t], prob[i, ti[i]].numpy(), rtol=1e-12)
        assert (np.diff(scores[t]) <= 0).all() and 0 < scores[t].sum() <= 1 + 1e-12
    written = np.zeros(V, bool)
    written[tokens] = True
    assert (ids[~written] == -1).all()
    # K = V returns every token once, scores sum to one
    ids_all, sc_all = orc.harvest_topk(logits[:1], tokens[:1], V)
    assert sorted(ids_all[tokens[0]].tolist()) == list(range(V))
    np.testing.assert_allclose(sc_all[tokens[0]].sum(), 1.0, rtol=1e-12)


def test_ties_and_repeated_tokens():
    logits = np.zeros((3, 8))
    logits[0, [6, 2, 4]] = 1.0                                     # three equal maxima: ids ascending
    logits[1, 7] = 2.0
    logits[2, 1] = 5.0
    ids, _ = orc.harvest_topk(logits, [3, 3, 0], 4)                # nodes 0 and 1 both carry token 3
    assert ids[3].tolist() == [7, 0, 1, 2]                         # the later node wins; then equal zeros by id
    assert ids[0].tolist() == [1, 0, 2, 3]
    ids0, _ = orc.harvest_topk(logits[:1], [3], 4)
    assert ids0[3].tolist() == [2, 4, 6, 0]
    # existing rows survive a later harvest that does not touch them
    ids2, sc2 = orc.harvest_topk(logits[2:], [5], 4, table_ids=ids, table_scores=np.ones((8, 4)))
    assert ids2[3].tolist() == [7, 0, 1, 2] and ids2[5].tolist() == [1, 0, 2, 3] and (sc2[3] == 1).all()
