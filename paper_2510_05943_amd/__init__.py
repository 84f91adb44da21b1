"""MI355X-native re-layout of intermediate RL rollout batches (the data dispatcher's hot path).

`binding` wraps the C-ABI library built from `csrc/`; `synth` draws the synthetic batches.
Importing the package does not load the library; the first call into `binding` does, and
fails loudly if the library has not been built.
"""
__all__ = ["binding", "synth"]
