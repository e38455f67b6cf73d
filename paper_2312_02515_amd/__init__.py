"""MI355X-native BatchLoRA multi-adapter LoRA linear operator (forward + backward).

`workloads` holds shapes and seeded input generators (no arithmetic of the
method).  `binding` is the thin ctypes layer over the C-ABI library
`libmlora.so`; importing it loads the library and fails loudly if it has not
been built (`python -c "import __graft_entry__ as g; g.build()"`).
"""
__all__ = ["workloads", "binding", "buildlib"]
