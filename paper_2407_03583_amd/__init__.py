"""MI355X-native exhaustive allocation search after Loki (HPDC'24).

`binding` wraps the C-ABI library (include/loki_alloc.h); `workloads` draws the
seeded synthetic inputs; `build` compiles the library for gfx950.
"""
