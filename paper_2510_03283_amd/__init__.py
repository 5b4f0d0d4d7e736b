"""MI355X-native hybrid iteration (prefill + decode + DPO fine-tune rows) of one decoder layer.

`synth` holds the seeded workload generator; `binding` loads the HIP library and exposes
its C-ABI entry points under the same names.  Importing the package loads neither.
"""
