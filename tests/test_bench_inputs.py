"""Inputs that bench.py builds for its optional legs, checked on the CPU with the oracle."""
import numpy as np

import bench
import synth
from oracle import model as M, serve as SV
from oracle.scheduler import Scheduler


def test_cycle_weights_make_every_stream_cycle_and_every_draft_right():
    """bench.cycle_weights (the upper-bound input of the speculative-decoding leg): the oracle's greedy stream after token t
    is t's successors inside its group of 16 ids, whatever the prompt; the speculative scheduler then accepts every draft
    once the stream has come round."""
    cfg = dict(synth.model_config("mini_gqa"), vocab=2496)
    W = M.Weights(cfg, bench.cycle_weights(cfg, synth.make_weights(cfg, 5)))
    r = dict(prompt=np.array([5, 900, 33], dtype=np.int32), max_new_tokens=40, temperature=0.0, top_k=0, top_p=1.0, seed=0)
    out = SV.generate_reference(cfg, W, r)
    assert out == [32 + (33 + 1 + i - 32) % 16 for i in range(40)]
    eng = dict(kv_block_size=16, kv_num_blocks=16, max_batch=2, max_seq_len=64, max_prefill_tokens=64, ring_slots=4, eos_token_id=-1, speculative=4)
    ev, sched = SV.serve(cfg, W, eng, [r])
    assert sched.outputs[0] == out
    assert sched.drafted == sched.accepted > 15 and sched.iteration < 30


def test_repetitive_prompts_keep_lengths_and_repeat():
    reqs = synth.make_workload("mini", 500, 3, n_requests=6)
    rep = synth.with_repetition(reqs, 500, 4)
    for a, b in zip(reqs, rep):
        assert len(a["prompt"]) == len(b["prompt"]) and b["prompt"].dtype == np.int32
        assert len(set(b["prompt"].tolist())) <= 6
