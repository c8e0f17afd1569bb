"""MI355X-native kernels for SwiftDiffusion's base-model hot path (arXiv 2407.02031).

The package is a thin binding over libswiftdiff.so (HIP kernels behind a C ABI, declared
in include/swiftdiff.h).  Attribute access loads the binding lazily so that the build
module can be imported before the library exists; using any entry point without the
built library raises ImportError — there is no CPU or torch fallback.
"""
import importlib

_BINDING_NAMES = {
    "lora_linear_fwd", "attention_fwd", "attn_block_fwd", "ff_block_fwd", "groupnorm_fwd",
    "spatial_transformer_fwd", "spatial_transformer_workspace_bytes", "multi_lora_linear_fwd",
    "lora_patch", "lora_unpatch", "timing_enable", "timing_collect", "timing_disable", "TIMING_TAGS", "PatchPlan", "Proj", "StackParams", "to_bf16", "SwiftDiffError",
    "SD_BF16", "SD_F32", "SD_EPI_NONE", "SD_EPI_GEGLU", "LIB_PATH", "EXPORTS", "lib",
}


def __getattr__(name):
    if name in _BINDING_NAMES or name == "binding":
        mod = importlib.import_module(".binding", __name__)
        return mod if name == "binding" else getattr(mod, name)
    raise AttributeError(name)
