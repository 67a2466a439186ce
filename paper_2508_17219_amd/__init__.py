"""MI355X-native segment-level prefix attention (TokenLake's cache-aware operation).

`workloads` draws seeded synthetic inputs; `binding` is the thin ctypes layer over the C-ABI
library built from `csrc/` (pool, plan, segment partial attention, causal block, LSE merge).
"""
