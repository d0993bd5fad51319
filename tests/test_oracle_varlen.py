"""Pins for the oracle's loss on right-padded batches of unequal length.

* full lengths reproduce the fixed-length loss bit for bit;
* truncation: the loss of a padded batch equals what the sequences give when each is run alone, cut to its own
  length (a separate evaluation with different shapes), combined as a mean over all loss positions;
* what sits in the padding does not matter (causal attention: a real token never looks at a later position);
* a planted off-by-one in the valid range or in the last position is caught by the truncation pin.
"""
import numpy as np
import pytest

import workloads as W
from oracle import zo
from oracle.model import copy_loss, embed, decoder_layer, head_loss
from oracle.precision import Precision
from small_workloads import MINI_LLAMA, MINI_OPT


def _setup(w, seed=3):
    lay = W.lora_layout(w)
    frozen = W.make_frozen_weights(w, 1234)
    masters = W.make_lora_masters(w, 99, b_std=0.02)
    lora = zo.split_factors(lay, masters.astype(np.float64))
    tokens, labels = W.make_tokens(w, seed), W.make_labels(w, seed)
    return frozen, lora, tokens, labels


CASES = [MINI_LLAMA, MINI_OPT, MINI_OPT.with_(loss_mode="next_token_all_pos"),
         MINI_LLAMA.with_(loss_mode="last_pos_label_subset", label_tokens=(3, 11))]


@pytest.mark.parametrize("w", CASES, ids=lambda w: f"{w.name}-{w.loss_mode}")
def test_full_lengths_equal_fixed_length_loss(w):
    frozen, lora, tokens, labels = _setup(w)
    for mode in ("exact", "f32"):
        prec = Precision(mode)
        a = copy_loss(w, frozen, lora, tokens, labels, prec)
        b = copy_loss(w, frozen, lora, tokens, labels, prec, lengths=np.full(w.E, w.S))
        assert a == b


@pytest.mark.parametrize("w", CASES, ids=lambda w: f"{w.name}-{w.loss_mode}")
def test_padded_batch_equals_truncated_single_sequences(w):
    frozen, lora, tokens, labels = _setup(w)
    prec = Precision("exact")
    lengths = np.array([w.S, max(2, w.S // 3)] + [max(2, w.S - 5)] * (w.E - 2))[:w.E]
    got = copy_loss(w, frozen, lora, tokens, labels, prec, lengths=lengths)
    # every sequence alone, cut to its own length: sum of its position losses and their number
    total, count = 0.0, 0
    for e in range(w.E):
        L = int(lengths[e])
        we = w.with_(E=1, S=L)
        le = copy_loss(we, frozen, lora, tokens[e:e + 1, :L], labels[e:e + 1], prec)
        n_pos = L - 1 if w.loss_mode == "next_token_all_pos" else 1
        total += le * n_pos
        count += n_pos
    assert abs(got - total / count) <= 1e-12 * abs(got)
    # planted mistakes: one position too many / too few, or the last slot instead of the last token
    h = embed(w, frozen, tokens, prec)
    for li, lw in enumerate(frozen["layers"]):
        h = decoder_layer(w, lw, li, h, lora, prec)
    for wrong in (lengths + (lengths < w.S), np.maximum(lengths - 1, 2), np.full(w.E, w.S)):
        if np.array_equal(wrong, lengths):
            continue
        bad = head_loss(w, frozen, h, tokens, labels, prec, lengths=wrong)
        assert abs(bad - total / count) > 1e-9 * abs(got)


@pytest.mark.parametrize("w", CASES[:3], ids=lambda w: f"{w.name}-{w.loss_mode}")
def test_padding_content_is_irrelevant(w):
    frozen, lora, tokens, labels = _setup(w)
    prec = Precision("f32")
    lengths = W.make_lengths(w, 5, pad_fraction=0.3)
    assert lengths.max() == w.S and lengths.min() >= 2
    a = copy_loss(w, frozen, lora, tokens, labels, prec, lengths=lengths)
    t2 = tokens.copy()
    rng = np.random.default_rng(0)
    for e in range(w.E):
        t2[e, lengths[e]:] = rng.integers(0, w.vocab, size=w.S - lengths[e])
    assert copy_loss(w, frozen, lora, t2, labels, prec, lengths=lengths) == a
