"""Workload shapes.  Names c1..c5 follow the order of the benchmark configurations:
c1 tiny fp32 plumbing case, c2 draft-model batched decode, c3 7B verify (N=3, gamma=4, S=512),
c4 wide 7B verify (N=16, gamma=6, S=2048, R=128), c5 13B verify (N=8, gamma=5, S=4096); c6 state-evaluator
shape, c7 / c8 the batch sweep past 128 rows.

Notation: N branches (the paper's n), gamma draft tokens per branch (the paper's k), S shared-prefix
tokens, R branch-private context tokens.
"""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class ModelCfg:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    dtype: str            # "fp32" or "bf16": storage type of weights and KV cache; "bf16w8": bf16 with the
                          # projection matrices as one-byte e4m3 codes + per-row scales
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def params(self):
        d, f, v = self.d_model, self.d_ff, self.vocab
        per_layer = 4 * d * d + 3 * d * f
        return self.n_layers * per_layer + v * d  # streamed per step: layers + LM head


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelCfg
    N: int
    gamma: int
    S: int
    R: int
    temperature: float      # target temperature
    q_kind: str             # "random" (softmax of N(0,1)/q_temp) or "perturbed" (target logits + noise)
    q_temp: float
    q_noise_std: float
    kv_protocol: str        # "true_prefix" or "synthetic"
    seed: int               # weights seed; seed+1 prefix/KV, +2 q logits, +3 draft draws, +4 uniforms
    R_min: int = -1         # >= 0: ragged private contexts, branch lengths seeded in [R_min, R]; < 0: all R

    def scaled(self, **kw):
        """Same workload with some fields replaced (e.g. fewer layers for a quick parity case)."""
        model_kw = {k: v for k, v in kw.items() if k in ModelCfg.__dataclass_fields__}
        wl_kw = {k: v for k, v in kw.items() if k not in model_kw}
        m = replace(self.model, **model_kw) if model_kw else self.model
        return replace(self, model=m, **wl_kw)


_TINY = ModelCfg(2, 256, 4, 64, 1024, 1024, "fp32")
_DRAFT = ModelCfg(2, 768, 12, 64, 3072, 32000, "bf16")
_7B = ModelCfg(32, 4096, 32, 128, 11008, 32000, "bf16")
_13B = ModelCfg(40, 5120, 40, 128, 13824, 32000, "bf16")

WORKLOADS = {
    "c1": Workload("c1", _TINY, N=3, gamma=4, S=64, R=0, temperature=0.8, q_kind="random", q_temp=0.8,
                   q_noise_std=0.0, kv_protocol="true_prefix", seed=1001),
    "c2": Workload("c2", _DRAFT, N=8, gamma=8, S=256, R=0, temperature=1.0, q_kind="random", q_temp=1.0,
                   q_noise_std=0.0, kv_protocol="true_prefix", seed=2001),
    "c3": Workload("c3", _7B, N=3, gamma=4, S=512, R=0, temperature=0.7, q_kind="random", q_temp=1.0,
                   q_noise_std=0.0, kv_protocol="synthetic", seed=3001),
    "c4": Workload("c4", _7B, N=16, gamma=6, S=2048, R=128, temperature=1.0, q_kind="random", q_temp=1.0,
                   q_noise_std=0.0, kv_protocol="synthetic", seed=4001),
    "c5": Workload("c5", _13B, N=8, gamma=5, S=4096, R=0, temperature=0.7, q_kind="perturbed", q_temp=0.7,
                   q_noise_std=0.5, kv_protocol="synthetic", seed=5001),
    # State-evaluator shape (Section 3.2: the evaluator scores different states, i.e. different prompts): no
    # shared prefix at all, every branch brings its own context of a different length.
    "c6": Workload("c6", _7B, N=8, gamma=4, S=0, R=1024, temperature=0.7, q_kind="random", q_temp=1.0,
                   q_noise_std=0.0, kv_protocol="synthetic", seed=6001, R_min=384),
    # Batch sweep past the matrix-core ridge (more branches than any search of the paper uses; the shapes of c4
    # otherwise): 384 and 768 rows per step.
    "c7": Workload("c7", _7B, N=64, gamma=6, S=2048, R=128, temperature=1.0, q_kind="random", q_temp=1.0,
                   q_noise_std=0.0, kv_protocol="synthetic", seed=7001),
    "c8": Workload("c8", _7B, N=128, gamma=6, S=2048, R=128, temperature=1.0, q_kind="random", q_temp=1.0,
                   q_noise_std=0.0, kv_protocol="synthetic", seed=8001),
}


def get_workload(name):
    return WORKLOADS[name]
