"""MI355X-native Power-SMC per-token step (vocabulary pass, ESS, systematic resampling, KV reindex).

The compute lives in the HIP library under csrc/ behind the C ABI declared in include/power_smc.h;
`binding` marshals arguments to it and nothing else.  Importing this package loads no native code.
"""
__all__ = ["binding", "synth"]
