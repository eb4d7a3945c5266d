"""Seeded synthetic inputs (model files, prompts, drafts) shared by the oracle
tests, the GPU parity tests and the benchmark.  Holds none of the method's
arithmetic."""
from .format import (ModelConfig, write_model, read_header, tensor_table, open_tensors,
                     bf16_to_f32, f32_to_bf16, build_lib, adapter_parameters)
from .workload import (TINY, LLAMA7B, LLAMA13B, prompt_tokens, corrupt_drafts,
                       session_corruption_p, embedding_prefix, draft_distributions)
