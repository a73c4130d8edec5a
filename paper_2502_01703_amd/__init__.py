"""MI355X-native QLESS gradient datastore and influence engine (HIP kernels behind a C ABI).

`synth` holds seeded synthetic inputs; `binding` is the thin ctypes layer over libqless.so.
Nothing here falls back to a CPU implementation: calling an entry point without the built
HIP library raises.
"""
