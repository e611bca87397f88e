"""The five benchmark shapes, as plain data.

Notation follows the paper (Section 3.1, 3.3): L_s system tokens come before
the image, L_v = N visual tokens, L_p prompt tokens after; the compression
target is L_vc tokens with merge proportion rho, so Stage I keeps
k_prune = L_vc(1+rho) tokens and Stage II merges k_prune - k_final of them.
"""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # 1-based config number; seeds are 10_000*index + image
    batch: int            # B
    n_vis: int            # N = L_v
    n_sys: int            # L_s  (tokens before the image)
    n_prompt: int         # L_p  (tokens after the image)
    n_heads: int          # H
    head_dim: int         # d_h
    dtype: str            # "f32" | "bf16" | "f16": storage type of Q,K,V,O,X
    k_prune: int          # L_vc (1 + rho)
    k_final: int          # L_vc
    rank: int             # planted rank of the hidden states
    spectrum: str         # "linspace" (10 -> 1) | "powerlaw" (s_i ~ i^-0.8, unit-RMS signal)
    noise: float          # std of the additive Gaussian noise on hidden states
    qkv_mode: str         # "iid": Q,K,V ~ N(0,1);  "proj": Q,K,V = X W_{q,k,v}, W ~ N(0, 1/D)
    lam: float = 0.5      # lambda of Eq. 3-8
    causal: int = 1

    @property
    def seq_len(self):
        return self.n_sys + self.n_vis + self.n_prompt

    @property
    def hidden(self):
        return self.n_heads * self.head_dim

    @property
    def n_merge(self):
        return self.k_prune - self.k_final

    def seed(self, image):
        return 10_000 * self.index + image

    def with_(self, **kw):
        return replace(self, **kw)


CONFIGS = {
    "tiny": Workload("tiny", 1, 1, 64, 4, 4, 4, 64, "f32", 16, 12, 8, "linspace", 0.01, "iid"),
    "llava7b_b1": Workload("llava7b_b1", 2, 1, 576, 36, 28, 32, 128, "bf16", 256, 192, 64,
                           "powerlaw", 0.05, "proj"),
    "llava7b_b64": Workload("llava7b_b64", 3, 64, 576, 36, 28, 32, 128, "bf16", 128, 64, 64,
                            "powerlaw", 0.05, "proj"),
    "hires_b8": Workload("hires_b8", 4, 8, 2880, 36, 28, 32, 128, "bf16", 960, 640, 128,
                         "powerlaw", 0.05, "proj"),
    "llava13b_b128": Workload("llava13b_b128", 5, 128, 576, 36, 28, 40, 128, "bf16", 96, 64, 64,
                              "powerlaw", 0.05, "proj"),
}


def get_config(name):
    return CONFIGS[name]
