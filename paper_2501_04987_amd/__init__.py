"""TreeKV hot path for MI355X (gfx950): attend -> score -> tree eviction -> compaction.

`binding` wraps the C-ABI library built from `csrc/`; `inputs` holds the seeded
synthetic stream generators.  There is no CPU fallback: importing `binding`
without the built HIP library raises.
"""
