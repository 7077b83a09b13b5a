"""Glue used by the tests only: turns the seeded inputs into the oracle's model object."""
import numpy as np

import mtmc_oracle as oracle
from paper_2511_20100_amd import inputs


def oracle_model(weights: inputs.Weights, max_positions: int = 4096, dtype=np.float32) -> oracle.Model:
    c = weights.cfg
    return oracle.Model(n_layers=c.n_layers, d_model=c.d_model, n_q_heads=c.n_q_heads,
                        n_kv_heads=c.n_kv_heads, head_dim=c.head_dim, d_ffn=c.d_ffn, vocab=c.vocab,
                        rms_eps=c.rms_eps, rope_base=c.rope_base, w=weights.f32,
                        max_positions=max_positions, dtype=dtype)


def dict_model(tensors, *, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab,
               rms_eps=1e-6, rope_base=10000.0, max_positions=64, dtype=np.float64) -> oracle.Model:
    return oracle.Model(n_layers=n_layers, d_model=d_model, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
                        head_dim=head_dim, d_ffn=d_ffn, vocab=vocab, rms_eps=rms_eps, rope_base=rope_base,
                        w=lambda name: tensors[name], max_positions=max_positions, dtype=dtype)


def small_cfg(**kw) -> inputs.ModelConfig:
    base = dict(n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=48, vocab=64,
                dtype="fp32")
    base.update(kw)
    return inputs.ModelConfig(**base)
