"""MI355X-native causal linear attention with a causal depthwise-conv branch.

The work is done by hand-written HIP kernels behind a C-ABI shared library
(``include/linattn.h``); ``binding`` marshals arguments to it and nothing else.
Importing this package does not load the library; the first call does, and it
raises if the library has not been built.
"""
