"""Size of the KV pool of the Churn workload: "60 % of peak demand". Oracle-side script: test infrastructure only.

The workload description fixes the pool only as a share of the peak demand. The reading taken here: every request
holds its worst-case block reservation (oracle.scheduler.blocks_needed, the admission rule of the scheduler) from
its arrival for prompt * 20 us + output * 2 ms (a fluid model of the service with an unlimited pool); the pool is
60 % of the peak of the summed reservations, and at least the largest single reservation (or that request could
never be admitted).

  python -m oracle.churn_pool            prints the pool size for the default Churn request set (seed 2001)

The printed number is what synth.configs holds as the Churn engine's kv_num_blocks; a test compares the two.
"""
import sys

from .scheduler import blocks_needed


def peak_block_demand(reqs, bs, step_s=2.0e-3, prefill_s_per_token=2.0e-5):
    ev = []
    for r in reqs:
        need = blocks_needed(len(r["prompt"]), r["max_new_tokens"], bs)
        t0 = r["arrival_s"]
        t1 = t0 + len(r["prompt"]) * prefill_s_per_token + r["max_new_tokens"] * step_s
        ev.append((t0, need))
        ev.append((t1, -need))
    ev.sort(key=lambda e: (e[0], e[1]))
    cur = peak = 0
    for _, dlt in ev:
        cur += dlt
        peak = max(peak, cur)
    return peak


def churn_pool_blocks(reqs, bs=16):
    largest = max(blocks_needed(len(r["prompt"]), r["max_new_tokens"], bs) for r in reqs)
    return int(max(-(-6 * peak_block_demand(reqs, bs) // 10), largest))


if __name__ == "__main__":
    import synth
    cfg = synth.model_config("churn")
    print(churn_pool_blocks(synth.make_workload("churn", cfg["vocab"], 2001), synth.engine_config("churn")["kv_block_size"]))
    sys.exit(0)
