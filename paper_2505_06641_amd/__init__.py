"""MI355X-native SneakPeek scoring and batch-aware greedy scheduling.

`workloads` draws seeded synthetic inputs; `binding` wraps the C-ABI library
built from `csrc/` (loaded on first use, never at import of this package).
"""
