"""The five synthetic workloads of the window-scoring benchmark.

They take the shapes of the paper's draft/target model pairs: speculative
windows of up to K = 10 drafted tokens (Table 5) over vocabularies the size of
the LLaMA-2 / LLaMA-3 / Qwen families the paper evaluates (Section 5.1), with
the drafter cost ratio gamma, tolerance epsilon and scale eta of Table 5 as
parameter defaults.  No model, dataset or benchmark item is involved: logits
are seeded random numbers (see generate.py).
"""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "f32" or "bf16": storage type of both logit tensors
    B: int                # windows per scoring call
    K: int                # drafted positions per window
    V: int                # vocabulary size
    verify: str           # "rejection" or "greedy"
    cost_ratio: float     # gamma of the Cost-Aware Speedup Reward
    M: int                # windows kept by the top-M selection (over all chunks)
    seed: int
    family: str           # logit recipe, see generate.py
    chunks: int = 1       # scoring calls per pass (B windows each)
    expected_accept: bool = False   # also run the normalised-probability pass
    prox_eps: float = 0.5
    prox_eta: float = 1.0
    seq_len: int = 0      # > 0: sequence mode, B sequences of seq_len teacher-forced positions

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def logit_bytes_per_window(self) -> int:
        """Algorithmic bytes: both logit rows of every position, read once."""
        return 2 * self.K * self.V * self.elem_bytes

    def scaled(self, B: int, M: int = None, chunks: int = None) -> "Workload":
        """Same recipe at a different window count (parity-test sizes)."""
        if M is None:
            M = max(1, min(self.M, B * (chunks or self.chunks) // 8))
        return replace(self, B=B, M=M, chunks=self.chunks if chunks is None else chunks)


WORKLOADS = {
    "tiny_f32": Workload("tiny_f32", "f32", 32, 4, 1000, "rejection", 0.05, 8, 0, "boosted"),
    "greedy_bf16_32k": Workload("greedy_bf16_32k", "bf16", 4096, 7, 32000, "greedy", 0.04, 512, 1,
                                "zipf"),
    "rejection_bf16_128k": Workload("rejection_bf16_128k", "bf16", 16384, 8, 128256, "rejection",
                                    0.03, 2048, 2, "zipf"),
    "twopass_f32_152k": Workload("twopass_f32_152k", "f32", 8192, 8, 152064, "rejection", 0.05,
                                 1024, 3, "tempered", expected_accept=True),
    "stream_bf16_128k": Workload("stream_bf16_128k", "bf16", 8192, 10, 128256, "rejection", 0.03,
                                 8192, 4000, "zipf", chunks=8),
}

# Sequence-mode ADAW (Algorithm 1): 64 responses of 2048 positions, every overlapping window of
# K = 10 scored from one pass over the rows.
WORKLOADS["sequence_bf16_128k"] = Workload("sequence_bf16_128k", "bf16", 64, 10, 128256, "rejection",
                                           0.03, 2048, 5, "zipf", seq_len=2048)

# order of the benchmark's configuration list: index 1 is the greedy 32K case
ORDER = ["tiny_f32", "greedy_bf16_32k", "rejection_bf16_128k", "twopass_f32_152k",
         "stream_bf16_128k"]
