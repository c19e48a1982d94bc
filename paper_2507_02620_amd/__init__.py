"""MI355X-native tree-verification stage of FlowSpec (hand-written HIP behind a C ABI).

`flowspec` is the thin binding over the library; `synth` draws the seeded synthetic inputs.
Nothing here falls back to a CPU or PyTorch implementation: without the built library the
binding raises.
"""
