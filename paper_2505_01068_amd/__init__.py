"""MI355X-native Interlaced-Mask attention (GsiT hot path): thin Python binding
over the C-ABI library built from csrc/.  The binding loads lazily so that the
input generator (`synth`) can be imported on machines without the built library;
any compute call without it raises."""

from . import synth  # noqa: F401


def __getattr__(name):
    if name in ("binding", "im_attention_fwd", "im_attention_bwd", "gsit_layer_fwd",
                "im_attention_sizes", "gsit_layer_sizes", "ImShape", "lib",
                "IM_IFM_FORWARD", "IM_IFM_BACKWARD", "IM_IEM", "IM_DENSE"):
        import importlib
        b = importlib.import_module(".binding", __name__)
        return b if name == "binding" else getattr(b, name)
    raise AttributeError(name)
