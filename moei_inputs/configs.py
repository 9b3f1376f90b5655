"""Workload shapes (the five benchmark configurations) as plain data.

Notation follows the paper (Sec. 4.3): L MoE layers, E routed experts per
layer, k experts per token; H hidden width, I expert intermediate width,
N traces in the EAMC, S HBM cache slots.
"""
from dataclasses import dataclass, replace

BASE_SEED = 240114361


@dataclass(frozen=True)
class Config:
    name: str
    cid: int            # enters the seed: stream = BASE_SEED + 1000*cid + purpose
    L: int
    E: int
    k: int
    n_shared: int
    H: int
    I: int
    wdtype: str         # "fp32" | "bf16" : storage type of weights and hidden states
    renorm: int         # 1 = gate weights renormalised over the k picks
    N: int              # traces in the EAMC
    S: int              # routed-expert cache slots
    prompt: int         # prefill tokens (only counted into the EAM, no FFN)
    decode: int         # decode tokens
    n_clusters: int     # activation groups; 0 = every trace has its own permutation
    zipf_s: float
    w_std: float = 0.02
    r_std: float = 0.05
    mix_noise: float = 0.2      # weight of the Dirichlet(0.3) noise in a preference row
    dirichlet_alpha: float = 0.3

    @property
    def LE(self) -> int:
        return self.L * self.E

    @property
    def expert_elems(self) -> int:
        return 3 * self.H * self.I

    @property
    def wbytes(self) -> int:
        return 4 if self.wdtype == "fp32" else 2

    @property
    def expert_bytes(self) -> int:
        return self.expert_elems * self.wbytes

    def scaled(self, **kw) -> "Config":
        """A copy with some fields replaced (reduced shapes for quick parity cases)."""
        return replace(self, **kw)


CONFIGS = {
    # Tiny MoE, fp32
    "C1": Config("C1", 1, L=4, E=8, k=2, n_shared=0, H=256, I=512, wdtype="fp32", renorm=1,
                 N=64, S=12, prompt=32, decode=16, n_clusters=4, zipf_s=1.2),
    # DeepSeek-V2-Lite-shaped
    "C2": Config("C2", 2, L=26, E=64, k=6, n_shared=2, H=2048, I=1408, wdtype="bf16", renorm=0,
                 N=1000, S=416, prompt=512, decode=128, n_clusters=20, zipf_s=1.1),
    # Mixtral-8x7B-shaped
    "C3": Config("C3", 3, L=32, E=8, k=2, n_shared=0, H=4096, I=14336, wdtype="bf16", renorm=1,
                 N=1000, S=96, prompt=256, decode=256, n_clusters=0, zipf_s=0.8),
    # DeepSeek-V2-shaped layer slice, resident pool
    "C4": Config("C4", 4, L=59, E=160, k=6, n_shared=2, H=5120, I=1536, wdtype="bf16", renorm=0,
                 N=10000, S=2048, prompt=0, decode=128, n_clusters=20, zipf_s=1.1),
    # batch sweep on the C2 shape, big EAMC, resident pool
    "C5": Config("C5", 5, L=26, E=64, k=6, n_shared=2, H=2048, I=1408, wdtype="bf16", renorm=0,
                 N=10000, S=1664, prompt=0, decode=64, n_clusters=20, zipf_s=1.1),
}


def get_config(name: str) -> Config:
    return CONFIGS[name]
