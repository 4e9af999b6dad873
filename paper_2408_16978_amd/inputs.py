"""Seeded synthetic inputs for the chunked-attention path.

This module holds none of the method's arithmetic: it only draws Q, K, V, dO
i.i.d. N(0,1) from a stated seed (one independent stream per tensor), rounds
them to the storage dtype, and names the benchmark configurations.  Both the
GPU tests / benchmark and the CPU oracle's tests read inputs from here; the
oracle is always fed the stored bits (bf16 or fp32) widened to fp64.
"""
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Config:
    name: str
    S: int
    chunk: int
    Hq: int
    Hkv: int
    D: int
    dtype: str          # "f32" | "bf16"
    kv_on_host: bool = False
    act_on_host: bool = False
    # backward from stored dS tiles (FPDT_BWD_STORE_DS): 5 executed GEMMs per chunk pair instead
    # of 7, for chunk^2 * Hq * 2 bytes of workspace
    store_ds: bool = False

    @property
    def u(self) -> int:
        return self.S // self.chunk

    @property
    def scale(self) -> float:
        return 1.0 / float(self.D) ** 0.5

    def flops_fwd(self) -> float:
        """Matmul FLOPs of the causal half (the paper's MFU convention, App. B)."""
        return 4.0 * self.D * self.Hq * self.S * (self.S + 1) / 2.0

    def flops_fwd_bwd(self) -> float:
        return 3.5 * self.flops_fwd()


# The five workloads: tiny fp32 parity case, GPT-2.7B head share, Llama-8B head
# share (GQA 4:1) at 256K resident and at 2M with K/V offload, Llama-70B head
# share (GQA 8:1) at 1M with K/V and activations offloaded.
CONFIGS = {
    "tiny": Config("tiny", 1024, 256, 2, 2, 64, "f32"),
    "gpt2p7b_64k": Config("gpt2p7b_64k", 65536, 8192, 4, 4, 80, "bf16"),
    # profiling-sized cut of the Llama-8B head share: one chunk, same kernels and tiles
    "llama8b_64k": Config("llama8b_64k", 65536, 65536, 8, 2, 128, "bf16"),
    "llama8b_256k": Config("llama8b_256k", 262144, 65536, 8, 2, 128, "bf16", store_ds=True),
    # the same workload in the one-launch-per-kernel form (dQ recomputes S and dP)
    "llama8b_256k_one_launch": Config("llama8b_256k_one_launch", 262144, 65536, 8, 2, 128, "bf16"),
    "llama8b_2m": Config("llama8b_2m", 2097152, 65536, 8, 2, 128, "bf16", kv_on_host=True, store_ds=True),
    "llama70b_1m": Config("llama70b_1m", 1048576, 65536, 8, 1, 128, "bf16", kv_on_host=True,
                          act_on_host=True, store_ds=True),
}

_TENSOR_IDS = {"Q": 0, "K": 1, "V": 2, "dO": 3}


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def normal(name: str, shape, seed: int, dtype: str, device="cpu") -> torch.Tensor:
    """N(0,1) tensor `name` (one of Q, K, V, dO) drawn from its own stream of
    `seed`, generated on `device`, rounded to `dtype`."""
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed) * 4 + _TENSOR_IDS[name])
    x = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    return x.to(torch_dtype(dtype))


def make_qkvdo(S, Hq, Hkv, D, dtype, seed, device="cpu"):
    """Q, dO [S,Hq,D] and K, V [S,Hkv,D]."""
    Q = normal("Q", (S, Hq, D), seed, dtype, device)
    K = normal("K", (S, Hkv, D), seed, dtype, device)
    V = normal("V", (S, Hkv, D), seed, dtype, device)
    dO = normal("dO", (S, Hq, D), seed, dtype, device)
    return Q, K, V, dO


def structured(kind: str, S, Hq, Hkv, D, dtype, seed, device="cpu"):
    """Q, K, V, dO with a score distribution that N(0,1) inputs do not produce (parity cases):
      "rising"  scores grow by ~10 along the key axis, so the running row maximum rises in
                nearly every key tile and the weight sits on the latest keys;
      "offset"  all of Q and K shifted by +3: scores ~ 9 sqrt(D) with a spread of a few units;
      "peaked"  Q and K drawn with sigma = 2.5: score spread ~6, a few keys carry each row.
    """
    Q, K, V, dO = (t.float() for t in make_qkvdo(S, Hq, Hkv, D, dtype, seed, device))
    if kind == "rising":
        ramp = torch.arange(S, device=Q.device, dtype=torch.float32) * (10.0 / S)
        Q[:, :, 0] = float(D) ** 0.5
        K[:, :, 0] += ramp[:, None]
    elif kind == "offset":
        Q += 3.0
        K += 3.0
    elif kind == "peaked":
        Q *= 2.5
        K *= 2.5
    else:
        raise ValueError(kind)
    dt = torch_dtype(dtype)
    return Q.to(dt), K.to(dt), V.to(dt), dO.to(dt)
