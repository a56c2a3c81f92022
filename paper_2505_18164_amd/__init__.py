"""libmdi: MI355X-native partition prefill/decode for model-distributed LLM inference.

`synth` (input recipes) imports without the HIP library; `mdi` (the ctypes
binding) loads the built shared object on first use and raises if it is absent.
"""
