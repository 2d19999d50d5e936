"""CPU oracle for the fused-MLP path and the attention subgraph.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the cpu_baseline leg of the benchmark may import this
package; the GPU library never does, and this package never imports the GPU library.
"""
from .oracle import (  # noqa: F401
    ACT_GELU_TANH,
    ACT_NONE,
    ACT_RELU,
    ACT_SIGMOID,
    build,
    layer_bf16,
    layer_f32,
    layer_f8,
    layer_i8,
    layer_i8_unfused,
    mlp,
    num_threads,
)
from .mha import SOFTMAX_FAST, SOFTMAX_STABLE, attention, attention_i8  # noqa: F401,E402
