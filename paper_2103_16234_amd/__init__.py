"""MI355X-native stride-1 forward direct convolution (NCHW fp32 / KCRS fp32).

`inputs` (seeded synthetic tensors and layer shapes) is importable anywhere; the HIP
binding is loaded on first use of `conv_fwd` and friends and fails loudly when the
compiled library is missing.
"""
from . import inputs  # noqa: F401

_BINDING_NAMES = ("conv_fwd", "conv_fwd_plan", "conv_fwd_planned", "conv_fwd_bias_relu", "conv_fwd_find", "conv_fwd_two_stage",
                  "conv_two_stage_workspace_bytes", "conv_fwd_plan_split_c", "conv_fwd_split_c", "conv_fwd_split_c_static", "conv_fwd_plan_request", "conv_set_stream", "conv_strerror",
                  "ConvPlan", "ConvError", "load_library", "library_path", "build_library")


def __getattr__(name):
    if name in _BINDING_NAMES or name == "binding" or name.startswith("CONV_"):
        import importlib
        mod = importlib.import_module(".binding", __name__)
        return mod if name == "binding" else getattr(mod, name)
    raise AttributeError(name)
