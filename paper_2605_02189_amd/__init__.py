"""MI355X-native stage-decode hot path of PipeMax (one pipeline stage, one GPU).

Nothing is imported eagerly: `synth_inputs` must stay importable without the
HIP library, and `binding` loads the C-ABI library and fails loudly without it.
"""
__all__ = ["binding", "synth_inputs", "build"]
