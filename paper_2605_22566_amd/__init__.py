"""Graph-KV attention for MI355X (gfx950): node paths of a wGraph resolved to
per-request block tables over a shared paged K/V pool, then prefill / decode
attention through those tables.  All compute runs in the HIP library behind the
C ABI declared in include/graphflow.h; this package only marshals arguments.

Submodules are imported on demand so that the input generators
(``paper_2605_22566_amd.workload``) can be used without the built library.
"""
__all__ = ["workload", "binding"]
