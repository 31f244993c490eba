"""MI355X-native allocation search for compound inference serving.

`workloads` draws the synthetic inputs; `jsv` is the binding of the C ABI
(include/jsv.h) implemented by csrc/ (HIP kernels + host planner);
`build` compiles it with hipcc.  Importing this package loads nothing.
"""
