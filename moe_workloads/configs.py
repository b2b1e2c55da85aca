"""Shapes of the five workloads (LM-1B MoE layer shapes: d=512, h=1024, k=4 flat or
2+2 hierarchical; Appendix C of the paper) and scaled-down variants for parity tests."""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class MoEShape:
    name: str
    T: int            # tokens in the batch (all time steps batched together, Section 3.1)
    d: int            # model width = expert input and output size
    h: int            # expert hidden size
    n: int            # experts (flat) or a*b (hierarchical)
    k: int            # experts per token (flat) or k_primary*k_secondary
    a: int = 0        # hierarchical: number of groups (0 = flat MoE)
    b: int = 0        # hierarchical: experts per group
    k_primary: int = 0
    k_secondary: int = 0
    expert_dtype: str = "bf16"   # "f32" or "bf16"
    w_importance: float = 0.1    # Appendix C: both loss weights 0.1
    w_load: float = 0.1
    zipf_beta: float = 0.0       # strength of the per-expert logit bias (0 = none)
    backward: bool = False
    seed: int = 170106538

    @property
    def A(self) -> int:
        return self.T * self.k

    @property
    def hierarchical(self) -> bool:
        return self.a > 0


CONFIGS = (
    MoEShape("cfg0_flat_f32", T=256, d=512, h=1024, n=16, k=4, expert_dtype="f32", seed=1701065380),
    MoEShape("cfg1_flat_bf16_n256", T=8192, d=512, h=1024, n=256, k=4, seed=1701065381),
    MoEShape("cfg2_flat_bf16_n2048", T=32768, d=512, h=1024, n=2048, k=4, seed=1701065382),
    MoEShape("cfg3_hier_bf16_64x256", T=65536, d=512, h=1024, n=64 * 256, k=4, a=64, b=256,
             k_primary=2, k_secondary=2, seed=1701065383),
    MoEShape("cfg4_flat_bf16_train_zipf", T=65536, d=512, h=1024, n=512, k=4, zipf_beta=0.27,
             backward=True, seed=1701065384),
)


def scaled_config(cfg: MoEShape, **overrides) -> MoEShape:
    """A copy of `cfg` with some sizes replaced (used for oracle-sized parity cases)."""
    out = replace(cfg, **overrides)
    if out.hierarchical:
        out = replace(out, n=out.a * out.b, k=out.k_primary * out.k_secondary)
    return out
