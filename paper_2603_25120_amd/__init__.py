"""MI355X-native pipeline-stage forward/backward for multimodal-LLM training.

The product is the HIP library `libmllm_stage.so` (C ABI in include/mllm_stage.h);
`paper_2603_25120_amd.binding` is its ctypes binding (argument marshalling only).
Importing this package does not load the library; `binding.lib()` does, and raises
if it has not been built (`python -m paper_2603_25120_amd.build`).
"""
__all__ = ["binding", "build"]
