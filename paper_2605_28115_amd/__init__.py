"""MI355X-native compact-prefill path of CIVIC: score -> select -> compact -> prefill attention -> KV write.

`paper_2605_28115_amd.binding` holds the Python names of the C ABI (include/civic.h) and loads
libcivic.so; `paper_2605_28115_amd.workloads` holds the seeded synthetic inputs;
`paper_2605_28115_amd.build` compiles the library in-tree.  The binding is imported lazily so
that the input generators can be used without the library.
"""

_API = ("civic_kept_count", "civic_select_workspace_bytes", "civic_compact_workspace_bytes",
        "civic_anchor_normalize", "civic_score", "civic_select", "civic_compact",
        "civic_prefill_attn", "civic_kv_write", "Grid", "CivicError")


def __getattr__(name):
    if name in _API:
        import importlib
        return getattr(importlib.import_module(__name__ + ".binding"), name)
    raise AttributeError(name)
