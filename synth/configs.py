"""The workload shapes: the five configurations of this build, the wide-beam recall shape, plus the
public-dataset shape of the paper (Implementation Details and Table 2)."""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class StepConfig:
    name: str
    B: int            # requests ("users") per batch
    d: int            # backbone hidden width
    e: int            # code-embedding / state width
    L: int            # semantic-ID levels
    V: int            # codebook size per level (equal radices)
    K: int            # beam size
    N: int            # catalog size (distinct items)
    dtype: str        # "f32" or "bf16"
    catalog: str      # "uniform" | "zipf1" | "zipf12"
    zipf_s: float = 0.0
    load_factor: float = 0.5
    w_std: float = 0.02
    queries: int = 0  # stand-alone verifier queries per call (Stress)

    @property
    def radices(self):
        return [self.V] * self.L

    def scaled(self, **kw):
        return replace(self, **kw)


CONFIGS = {
    "tiny": StepConfig("tiny", B=4, d=64, e=64, L=3, V=256, K=4, N=10_000,
                       dtype="f32", catalog="uniform"),
    "serving": StepConfig("serving", B=256, d=512, e=128, L=3, V=256, K=20,
                          N=1_000_000, dtype="bf16", catalog="zipf1", zipf_s=1.1),
    "wide": StepConfig("wide", B=1024, d=1024, e=128, L=4, V=1024, K=50,
                       N=10_000_000, dtype="bf16", catalog="zipf12", zipf_s=1.2),
    "stress": StepConfig("stress", B=0, d=0, e=0, L=3, V=4096, K=0,
                         N=100_000_000, dtype="bf16", catalog="uniform",
                         queries=4_000_000),
    "large": StepConfig("large", B=4096, d=2048, e=128, L=3, V=4096, K=100,
                        N=50_000_000, dtype="bf16", catalog="zipf1", zipf_s=1.1),
    # recall setting (Sec. 1, Table 1: beam 512; up to 1000 in item retrieval): the beam is wider
    # than anything that stays on chip, K*K = 262144 candidates per request are verified
    "recall": StepConfig("recall", B=64, d=1024, e=128, L=3, V=4096, K=512,
                         N=20_000_000, dtype="bf16", catalog="zipf1", zipf_s=1.1),
    # paper's public setting: L=3, T_l=512, beam 10, logit head 1024 wide; the
    # catalog sizes are the item counts of its three datasets (Table 2).
    "paper_yelp": StepConfig("paper_yelp", B=64, d=1024, e=128, L=3, V=512, K=10,
                             N=11_383, dtype="bf16", catalog="uniform"),
    "paper_beauty": StepConfig("paper_beauty", B=64, d=1024, e=128, L=3, V=512, K=10,
                               N=57_288, dtype="bf16", catalog="uniform"),
    "paper_games": StepConfig("paper_games", B=64, d=1024, e=128, L=3, V=512, K=10,
                              N=33_614, dtype="bf16", catalog="uniform"),
}


def get_config(name):
    return CONFIGS[name]
