"""MI355X-native embedding hot path of Persia-style hybrid recommender training.

`workload` generates seeded synthetic inputs (numpy only); `binding` is the thin
ctypes layer over the C-ABI library built from `csrc/` (needs torch + a GPU to run).
"""
