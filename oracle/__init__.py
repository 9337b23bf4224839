"""CPU oracle of the Blink serving step. TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy implementation of what the on-GPU serving step computes: the
Philox4x32-10 generator, the sampler, the decoder-only transformer (dense, cached and paged
variants), the FCFS continuous-batching scheduler with paged-KV accounting, and the
whole serving loop. Only tests, the smoke check and the cpu_baseline leg of the benchmark
may import it. It shares no code with the HIP path and never imports it; the product path
never routes through it.
"""
