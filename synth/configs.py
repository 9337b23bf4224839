"""Model and engine configurations of the five synthetic workloads.

Names: tiny, churn, llama3_8b, sched_stress (the interference run reuses llama3_8b).
dtype: 0 = fp32 weights and KV, 1 = bf16 weights and KV.
"""

MODEL_CONFIGS = {
    "tiny": dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=1024,
                 vocab=4096, dtype=0, rms_eps=1e-5, rope_theta=10000.0),
    "churn": dict(n_layers=8, d_model=1024, n_q_heads=16, n_kv_heads=16, head_dim=64, d_ffn=4096,
                  vocab=32000, dtype=1, rms_eps=1e-5, rope_theta=10000.0),
    "llama3_8b": dict(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
                      d_ffn=14336, vocab=128256, dtype=1, rms_eps=1e-5, rope_theta=500000.0),
    "sched_stress": dict(n_layers=1, d_model=128, n_q_heads=2, n_kv_heads=2, head_dim=64, d_ffn=512,
                         vocab=8192, dtype=0, rms_eps=1e-5, rope_theta=10000.0),
    # small GQA bf16 model used by parity tests only (several tiles, ragged tails, fast oracle)
    "mini_gqa": dict(n_layers=3, d_model=384, n_q_heads=6, n_kv_heads=2, head_dim=64, d_ffn=832,
                     vocab=2500, dtype=1, rms_eps=1e-5, rope_theta=500000.0),
    "mini_gqa128": dict(n_layers=2, d_model=512, n_q_heads=4, n_kv_heads=1, head_dim=128, d_ffn=1152,
                        vocab=3001, dtype=1, rms_eps=1e-5, rope_theta=500000.0),
    # wide FFN / vocabulary: the streaming GEMM takes 2 resp. 4 weight tiles per workgroup at these widths
    "mini_wide2": dict(n_layers=1, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=6400,
                       vocab=13001, dtype=1, rms_eps=1e-5, rope_theta=10000.0),
    "mini_wide4": dict(n_layers=1, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=12288,
                       vocab=24601, dtype=1, rms_eps=1e-5, rope_theta=10000.0),
    # the Churn model's shape (multi-head attention: one q head per kv head) with two layers instead of eight
    "mini_churn": dict(n_layers=2, d_model=1024, n_q_heads=16, n_kv_heads=16, head_dim=64, d_ffn=4096,
                       vocab=32000, dtype=1, rms_eps=1e-5, rope_theta=10000.0),
    # six and eight q heads per kv head
    "mini_g6": dict(n_layers=2, d_model=384, n_q_heads=6, n_kv_heads=1, head_dim=128, d_ffn=640,
                    vocab=1900, dtype=1, rms_eps=1e-5, rope_theta=10000.0),
    "mini_g8": dict(n_layers=2, d_model=512, n_q_heads=16, n_kv_heads=2, head_dim=64, d_ffn=768,
                    vocab=2100, dtype=1, rms_eps=1e-5, rope_theta=500000.0),
    # eight kv heads in one small layer: enough (sequence, chunk, kv head) items of decode attention at 40 sequences that
    # workgroups take items beyond their first two
    "mini_kv8": dict(n_layers=1, d_model=256, n_q_heads=16, n_kv_heads=8, head_dim=64, d_ffn=512,
                     vocab=1500, dtype=1, rms_eps=1e-5, rope_theta=10000.0),
    # the head configuration of the llama3_8b shape (32 q / 8 kv heads of 128) in one narrow layer: decode attention at
    # the full head count with enough sequences that the scheduler hands out whole contexts by itself
    "mini_heads32": dict(n_layers=1, d_model=512, n_q_heads=32, n_kv_heads=8, head_dim=128, d_ffn=512,
                         vocab=1024, dtype=1, rms_eps=1e-5, rope_theta=500000.0),
    # mixture of experts: d_ffn is the width of one expert
    "mini_moe": dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=96, n_experts=8, n_active=2,
                     vocab=1500, dtype=1, rms_eps=1e-5, rope_theta=10000.0),
    # sixteen experts, four active, wide enough that a prefill iteration gives an expert more than 64 tokens
    "mini_moe16": dict(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=160, n_experts=16, n_active=4,
                       vocab=2100, dtype=1, rms_eps=1e-5, rope_theta=10000.0),
    # the shape of the paper's mixture-of-experts model (30 B parameters, 3 B active per token): 128 experts of width 768, 8 active
    "moe_30b_a3b": dict(n_layers=48, d_model=2048, n_q_heads=32, n_kv_heads=4, head_dim=128, d_ffn=768, n_experts=128, n_active=8,
                        vocab=151936, dtype=1, rms_eps=1e-6, rope_theta=1000000.0),
}

# churn: the pool is "60 % of peak demand" of its default request set (256 requests, seed 2001), a number written by
# `python -m oracle.churn_pool` (a test keeps the two in step)
ENGINE_CONFIGS = {
    "tiny": dict(kv_block_size=16, kv_num_blocks=256, max_batch=8, max_seq_len=128,
                 max_prefill_tokens=8192, ring_slots=64, eos_token_id=-1),
    "churn": dict(kv_block_size=16, kv_num_blocks=297, max_batch=64, max_seq_len=2048 + 256,
                  max_prefill_tokens=8192, ring_slots=512, eos_token_id=-1),
    "llama3_8b": dict(kv_block_size=16, kv_num_blocks=32768, max_batch=256, max_seq_len=4096 + 1024,
                      max_prefill_tokens=8192, ring_slots=2048, eos_token_id=-1),
    "sched_stress": dict(kv_block_size=16, kv_num_blocks=65536, max_batch=512, max_seq_len=64,
                         max_prefill_tokens=8192, ring_slots=4096, eos_token_id=-1),
    "mini_gqa": dict(kv_block_size=16, kv_num_blocks=96, max_batch=6, max_seq_len=160,
                     max_prefill_tokens=256, ring_slots=32, eos_token_id=-1),
    "mini_gqa128": dict(kv_block_size=16, kv_num_blocks=64, max_batch=5, max_seq_len=200,
                        max_prefill_tokens=300, ring_slots=16, eos_token_id=-1),
    "mini_wide2": dict(kv_block_size=16, kv_num_blocks=400, max_batch=64, max_seq_len=160,
                       max_prefill_tokens=512, ring_slots=128, eos_token_id=-1),
    "mini_wide4": dict(kv_block_size=16, kv_num_blocks=400, max_batch=64, max_seq_len=160,
                       max_prefill_tokens=512, ring_slots=128, eos_token_id=-1),
    "mini_churn": dict(kv_block_size=16, kv_num_blocks=160, max_batch=8, max_seq_len=1200,
                       max_prefill_tokens=1536, ring_slots=32, eos_token_id=-1),
    "mini_g6": dict(kv_block_size=16, kv_num_blocks=96, max_batch=6, max_seq_len=700,
                    max_prefill_tokens=700, ring_slots=32, eos_token_id=-1),
    "mini_g8": dict(kv_block_size=16, kv_num_blocks=96, max_batch=6, max_seq_len=700,
                    max_prefill_tokens=700, ring_slots=32, eos_token_id=-1),
    "mini_kv8": dict(kv_block_size=16, kv_num_blocks=3200, max_batch=40, max_seq_len=1300,
                     max_prefill_tokens=4096, ring_slots=64, eos_token_id=-1),
    "mini_heads32": dict(kv_block_size=16, kv_num_blocks=1400, max_batch=176, max_seq_len=2200,
                         max_prefill_tokens=8192, ring_slots=256, eos_token_id=-1),
    "mini_moe": dict(kv_block_size=16, kv_num_blocks=96, max_batch=6, max_seq_len=160,
                     max_prefill_tokens=256, ring_slots=32, eos_token_id=-1),
    "mini_moe16": dict(kv_block_size=16, kv_num_blocks=400, max_batch=48, max_seq_len=700,
                       max_prefill_tokens=900, ring_slots=128, eos_token_id=-1),
    "moe_30b_a3b": dict(kv_block_size=16, kv_num_blocks=32768, max_batch=256, max_seq_len=4096 + 1024,
                        max_prefill_tokens=8192, ring_slots=2048, eos_token_id=-1),
}


def model_config(name):
    return dict(MODEL_CONFIGS[name])


def engine_config(name):
    return dict(ENGINE_CONFIGS[name])
