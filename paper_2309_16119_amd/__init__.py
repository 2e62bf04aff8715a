"""MI355X-native ModuLoRA linear layer: HIP kernels behind a C ABI, plus this thin binding.

    from paper_2309_16119_amd import modulora_fwd, modulora_bwd_input, modulora_bwd_lora

The binding (and with it libmodulora.so) is loaded on first use of one of its names,
so that `paper_2309_16119_amd.synth` (input generators) can be imported on its own.
"""
_BINDING_NAMES = (
    "QWeight", "ModuloraError", "modulora_status_string", "modulora_workspace_bytes",
    "modulora_dequant", "modulora_fwd", "modulora_bwd_input", "modulora_bwd_lora", "modulora_adamw", "modulora_quantize_rtn",
    "modulora_profile_begin", "modulora_profile_end", "lib", "LIB_PATH",
)
__all__ = list(_BINDING_NAMES) + ["ModuLoRALinear", "LPLoRAFunction", "FusedAdapterAdamW"]


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    if name in ("ModuLoRALinear", "LPLoRAFunction", "FusedAdapterAdamW"):
        from . import nn
        return getattr(nn, name)
    raise AttributeError(name)
