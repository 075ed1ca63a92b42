"""Model / drafter / tree shapes.

The five benchmark shapes follow the workloads of the paper's experiment
setup (targets of Llama-3-8B and Llama-2-13B shape, tree width 10, 60 draft
tokens, depth 6 or 7: section 4.1 "Implementations") with random weights in
place of trained checkpoints; the `t_*` entries are reduced shapes used only
by parity tests.
"""
from dataclasses import dataclass, asdict, replace

DTYPE_F32, DTYPE_BF16, DTYPE_F16 = 0, 1, 2
DTYPE_NAME = {DTYPE_F32: "f32", DTYPE_BF16: "bf16", DTYPE_F16: "f16"}


@dataclass(frozen=True)
class ModelConfig:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float
    rope_theta: float
    dtype: int                       # storage dtype of weights / GEMM operands
    n_specialists: int               # S
    positions_per_specialist: int    # n  (section 3.2: PosS-n)
    fc_bias: int
    top_k: int                       # tree width k
    depth: int                       # L
    total_tokens: int                # N draft nodes; the tree has N+1 rows
    max_seq: int
    kv_page_tokens: int
    n_prompt: int
    n_new: int
    weight_seed: int = 2506
    prompt_seed: int = 3566
    norm_gain_jitter: float = 0.0    # 0 => RMSNorm gains are exactly 1
    kv_page_order: int = 0           # physical page order of the KV caches (layout tests)

    @property
    def tree_rows(self):
        return self.total_tokens + 1

    @property
    def pool_size(self):
        return self.top_k + (self.depth - 1) * self.top_k * self.top_k

    def dict(self):
        return asdict(self)

    def with_(self, **kw):
        return replace(self, **kw)


def _llama3_8b(name, S, n, depth, total, n_prompt, n_new, max_seq):
    return ModelConfig(name=name, n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=8,
                       head_dim=128, d_ffn=14336, vocab=128256, rms_eps=1e-5,
                       rope_theta=500000.0, dtype=DTYPE_BF16, n_specialists=S,
                       positions_per_specialist=n, fc_bias=1, top_k=10, depth=depth,
                       total_tokens=total, max_seq=max_seq, kv_page_tokens=64,
                       n_prompt=n_prompt, n_new=n_new)


CONFIGS = {
    # C0: tiny fp32 reference shape
    "c0_tiny_f32": ModelConfig(
        name="c0_tiny_f32", n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64,
        d_ffn=688, vocab=4096, rms_eps=1e-5, rope_theta=10000.0, dtype=DTYPE_F32,
        n_specialists=3, positions_per_specialist=2, fc_bias=1, top_k=4, depth=6,
        total_tokens=24, max_seq=512, kv_page_tokens=64, n_prompt=64, n_new=32),
    # C1: Llama-3-8B shape, 3 specialists x 2 positions
    "c1_llama3_8b_3x2": _llama3_8b("c1_llama3_8b_3x2", 3, 2, 6, 60, 512, 256, 1024),
    # C2: Llama-3-8B shape, 6 specialists x 1 position
    "c2_llama3_8b_6x1": _llama3_8b("c2_llama3_8b_6x1", 6, 1, 6, 60, 512, 256, 1024),
    # C3: Llama-2-13B shape fp16
    "c3_llama2_13b_3x2": ModelConfig(
        name="c3_llama2_13b_3x2", n_layers=40, d_model=5120, n_q_heads=40, n_kv_heads=40,
        head_dim=128, d_ffn=13824, vocab=32000, rms_eps=1e-5, rope_theta=10000.0,
        dtype=DTYPE_F16, n_specialists=3, positions_per_specialist=2, fc_bias=1, top_k=10,
        depth=6, total_tokens=60, max_seq=1536, kv_page_tokens=64, n_prompt=1024, n_new=256),
    # C4: long context on the 8B shape, depth 7, 80 draft tokens
    "c4_llama3_8b_long": _llama3_8b("c4_llama3_8b_long", 3, 2, 7, 80, 8192, 128, 8576),
    # ---- reduced shapes for parity tests (not benchmark lines) ----
    "t_mid_bf16": ModelConfig(
        name="t_mid_bf16", n_layers=3, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64,
        d_ffn=1408, vocab=8192, rms_eps=1e-5, rope_theta=500000.0, dtype=DTYPE_BF16,
        n_specialists=3, positions_per_specialist=2, fc_bias=1, top_k=10, depth=6,
        total_tokens=60, max_seq=512, kv_page_tokens=64, n_prompt=150, n_new=24,
        norm_gain_jitter=0.1),
    "t_mid_f16": ModelConfig(
        name="t_mid_f16", n_layers=2, d_model=640, n_q_heads=5, n_kv_heads=5, head_dim=128,
        d_ffn=1728, vocab=5000, rms_eps=1e-5, rope_theta=10000.0, dtype=DTYPE_F16,
        n_specialists=2, positions_per_specialist=3, fc_bias=1, top_k=10, depth=7,
        total_tokens=80, max_seq=512, kv_page_tokens=64, n_prompt=131, n_new=16,
        norm_gain_jitter=0.1),
    "t_tiny_f32_6x1": ModelConfig(
        name="t_tiny_f32_6x1", n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64,
        d_ffn=688, vocab=4096, rms_eps=1e-5, rope_theta=10000.0, dtype=DTYPE_F32,
        n_specialists=6, positions_per_specialist=1, fc_bias=1, top_k=4, depth=6,
        total_tokens=24, max_seq=512, kv_page_tokens=64, n_prompt=70, n_new=24,
        norm_gain_jitter=0.1),
}


def get_config(name, **overrides):
    cfg = CONFIGS[name]
    return cfg.with_(**overrides) if overrides else cfg
