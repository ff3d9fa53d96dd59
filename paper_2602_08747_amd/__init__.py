"""MI355X-native batched latency estimate / drop decision / survivor compaction
(the data-parallel hot path of PARD's proactive request dropping).

`binding` wraps the C-ABI of libpard.so; `workloads` draws seeded synthetic inputs;
`build` compiles the HIP sources.  Importing the package loads nothing.
"""
__all__ = ["binding", "build", "workloads"]
