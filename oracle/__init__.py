"""CPU oracle for the paged-KV decode-attention path.

TEST INFRASTRUCTURE ONLY.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the product package
never does, and this package never imports the product package.
"""
from .paged_attention import (  # noqa: F401
    build_oracle,
    paged_attention,
    paged_attention_probs,
    paged_attention_kv8,
    fp8e4m3_to_f64,
    oracle_threads,
    bits_of,
    widen_bits,
)
from .layerstack import layer_gemm_bf16, round_to_bf16_bits, layerstack_layer  # noqa: F401
from .working_set import block_bytes, iteration_working_set_bytes, max_resident_batches  # noqa: F401
from .alg1_model import blocks_used, fetches_in_flight  # noqa: F401
