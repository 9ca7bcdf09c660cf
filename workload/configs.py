"""Named workload presets: the five benchmark configurations, a ten-head variant, and reduced-depth test cuts.

Shapes follow a Llama-style decoder-only model (the paper's CodeLlama-7b base, Section
III-B / IV-A) with Medusa-style draft heads on the last hidden state. The paper fixes none
of top-k, tree size or head count for a step beyond "10 heads" (Section IV-A); the numbers
here are the benchmark's.
"""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    n_medusa: int          # H: number of draft heads
    topk: int              # k: candidates kept per head
    dtype: str             # "f32" or "bf16": storage type of weights / KV on the device
    rope_theta: float
    rms_eps: float = 1e-5

    def with_layers(self, n_layers: int) -> "ModelShape":
        return replace(self, n_layers=n_layers)


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelShape
    tree_nodes: int        # T, root included
    batch: int
    prompt_len: int
    decode_steps: int
    kv_cap: int
    stop_frac: float = 0.2
    zipf_s: float = 1.1


_TINY = ModelShape(2, 256, 4, 64, 688, 1024, 3, 4, "f32", 1e4)
_7B = ModelShape(32, 4096, 32, 128, 11008, 32016, 4, 10, "bf16", 1e6)
_13B = ModelShape(40, 5120, 40, 128, 13824, 32016, 5, 10, "bf16", 1e6)
_7B_H10 = ModelShape(32, 4096, 32, 128, 11008, 32016, 10, 10, "bf16", 1e6)     # the paper's ten heads (Section IV-A)

PRESETS = {
    # configs[0]: the small case the oracle finishes in seconds
    "tiny": Workload("tiny", _TINY, 16, 1, 64, 32, 256),
    # configs[1]: the configuration the headline metric is quoted on
    "7b": Workload("7b", _7B, 64, 1, 512, 256, 2048),
    # configs[2]: long context
    "7b-long": Workload("7b-long", _7B, 64, 1, 16384, 128, 16896),
    # configs[3]: batched, ragged KV lengths in [1024, 4096]
    "7b-batch8": Workload("7b-batch8", _7B, 32, 8, 0, 64, 4096 + 64 * 5),
    # configs[4]
    "13b": Workload("13b", _13B, 128, 1, 4096, 128, 4096 + 128 * 6),
    # beyond the five benchmark configurations: ten draft heads and the largest tree the library takes
    "7b-h10": Workload("7b-h10", _7B_H10, 256, 1, 512, 128, 2048),
}


def preset(name: str, n_layers: int | None = None) -> Workload:
    """Look a preset up; `n_layers` cuts the depth (same width) for oracle-sized parity runs."""
    w = PRESETS[name]
    if n_layers is not None:
        w = replace(w, name=f"{w.name}-L{n_layers}", model=w.model.with_layers(n_layers))
    return w
