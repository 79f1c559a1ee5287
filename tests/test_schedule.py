"""The multi-stage schedule (Section 3.2, Figure 1) with the counts of Section 4.1, and the order of calls
the harness makes.  CPU only: the library is replaced by a recorder."""
import pytest

from paper_2011_13635_amd import schedule as S


def test_schedule_counts_of_the_paper():
    # Section 4.1: k = 4 stages, 3 layers per stage for BERT-Base and 6 for BERT-Large;
    # Section 4.2: 200 000 steps per stage, 200 000 retraining steps, 1 000 000 in total
    for n_layers, per in ((12, 3), (24, 6)):
        st = S.mslt_schedule(n_layers, 4, 200_000, 200_000, 0.00088, 0.0001)
        assert [s.name for s in st] == ["stage1", "stage2", "stage3", "stage4", "retrain"]
        assert [(s.frozen, s.trainable) for s in st] == [(0, per), (per, per), (2 * per, per), (3 * per, per), (0, n_layers)]
        assert [s.train_embeddings for s in st] == [True, False, False, False, True]
        assert [s.grow_first for s in st] == [0, per, per, per, 0]
        assert sum(s.steps for s in st) == 1_000_000
        assert st[0].lr == 0.00088 and st[-1].lr == 0.0001
    with pytest.raises(ValueError):
        S.mslt_schedule(12, 5, 1, 1, 1e-3)


def test_warmup_is_linear_then_flat():
    assert S.warmup_factor(0, 10_000) == pytest.approx(1e-4)
    assert S.warmup_factor(4_999, 10_000) == pytest.approx(0.5)
    assert S.warmup_factor(9_999, 10_000) == 1.0
    assert S.warmup_factor(123_456, 10_000) == 1.0
    assert S.warmup_factor(0, 0) == 1.0


class Recorder:
    def __init__(self):
        self.calls = []

    def mslt_grow(self, present, new):
        self.calls.append(("grow", present, new))

    def mslt_train_step(self, f, k, emb, batch, opt):
        self.calls.append(("step", f, k, bool(emb), batch, round(opt, 9)))
        return float(len(self.calls))


def test_harness_call_order():
    st = S.mslt_schedule(4, 2, 2, 1, 0.01, 0.001)
    rec = Recorder()
    losses = S.run_schedule(rec, st, next_batch=lambda g: g, make_opt=lambda lr: lr, warmup_steps=4)
    assert rec.calls == [
        ("step", 0, 2, True, 0, 0.0025), ("step", 0, 2, True, 1, 0.005),
        ("grow", 2, 2),
        ("step", 2, 2, False, 2, 0.0075), ("step", 2, 2, False, 3, 0.01),
        ("step", 0, 4, True, 4, 0.001),
    ]
    assert [len(x) for x in losses] == [2, 2, 1]


def test_last_tenth_of_the_steps_on_long_sequences():
    # Section 4.2: the last 10 % of the steps use sequences of 512
    st = S.mslt_schedule(12, 4, 200_000, 200_000, 0.00088, 0.0001)
    out = S.long_sequence_tail(st, 0.10, 512)
    assert sum(s.steps for s in out) == 1_000_000
    assert [(s.name, s.steps, s.seq_len) for s in out[-2:]] == [("retrain", 100_000, 0), ("retrain-long", 100_000, 512)]
    assert [s.seq_len for s in out[:-1]] == [0] * 5 and out[-1].grow_first == 0
    # a tail that swallows whole entries and splits an earlier one; growth happens once, before the first half
    out = S.long_sequence_tail(S.mslt_schedule(4, 2, 10, 4, 0.01), 0.5, 64)
    assert [(s.name, s.steps, s.seq_len, s.grow_first) for s in out] == [
        ("stage1", 10, 0, 0), ("stage2", 2, 0, 2), ("stage2-long", 8, 64, 0), ("retrain", 4, 64, 0)]
    rec = Recorder()
    S.run_schedule(rec, out, next_batch=lambda g, stage: (g, stage.seq_len), make_opt=lambda lr: lr)
    assert rec.calls[10] == ("grow", 2, 2)
    assert [c[4] for c in rec.calls if c[0] == "step"][11:14] == [(11, 0), (12, 64), (13, 64)]
