"""MI355X-native variable-length packed self-attention (forward and backward).

The compute lives in a C-ABI shared library built from csrc/ (hand-written HIP for
gfx950); `binding` marshals arguments to it and `workloads` generates seeded inputs.
"""
from . import workloads  # noqa: F401


def __getattr__(name):
    # The binding loads the HIP library; import it lazily so CPU-only tools can use workloads.
    if name in ("binding", "varlen_attn_fwd", "varlen_attn_bwd", "VarlenAttnError"):
        import importlib
        b = importlib.import_module(".binding", __name__)
        return b if name == "binding" else getattr(b, name)
    raise AttributeError(name)
