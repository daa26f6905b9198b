"""MI355X-native residual-expanded quantized layer (PIPE, arXiv 2311.15806).

`workloads` (seeded synthetic inputs) imports without the HIP library;
everything else comes from `binding`, which needs libpipe_hip.so and raises if
it is missing.
"""
from . import workloads  # noqa: F401

_BINDING_NAMES = (
    "Expansion", "PipeError", "pipe_expand", "pipe_expand_with_operator", "pipe_expansion_order", "pipe_forward", "pipe_forward_acc",
    "pipe_forward_conv2d", "pipe_mlp_forward", "pipe_chain_forward", "pipe_chain_forward_conv", "pipe_set_kernel", "pipe_timing_enable", "pipe_timing_read", "PIPE_ACT_NONE", "PIPE_ACT_GELU", "PIPE_ACT_SILU_GATED", "PIPE_ACT_RELU",
)


def __getattr__(name):
    if name in _BINDING_NAMES or name == "binding":
        import importlib
        b = importlib.import_module(__name__ + ".binding")
        return b if name == "binding" else getattr(b, name)
    raise AttributeError(name)
