"""DynamicKV prefill-time KV compression on MI355X: HIP kernels behind a C ABI.

`workloads` draws the seeded synthetic inputs; `dkv` is the thin binding over
libdkv.so (loaded on first use, never at import of this package).
"""
