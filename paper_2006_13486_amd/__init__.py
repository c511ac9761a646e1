"""MI355X-native RBGP4 sparse x dense product (O = W_s x I).

`workloads` holds the workload table and seeded synthetic inputs; `binding`
is the thin ctypes layer over the C-ABI library (loaded on first use)."""
