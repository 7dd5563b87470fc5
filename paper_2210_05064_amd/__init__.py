"""VER learner step on MI355X: ctypes binding over the HIP C-ABI library.

`binding` loads the built library and fails loudly when it is missing;
`workloads` draws seeded synthetic rollouts; `build` compiles the library.
Nothing is imported eagerly so that CPU-only tools can use `workloads`.
"""
