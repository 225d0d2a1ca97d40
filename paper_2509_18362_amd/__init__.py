"""MI355X-native FastMTP draft loop: HIP kernels behind a C ABI, plus a thin ctypes binding.

`synth` (seeded inputs) has no dependency on the compiled library; `binding` loads
libmtp_draft.so and fails loudly when it is missing.
"""
