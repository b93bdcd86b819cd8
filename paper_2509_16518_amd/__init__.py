"""MI355X-native forward kernel for fine-grained sparse attention (FG-Attn, Sec. 4.1-4.2).

Sub-modules:
  fgattn     -- thin ctypes binding over the C-ABI library (libfgattn.so); every step of
                the hot path runs in the library's HIP kernels.
  workloads  -- seeded synthetic inputs (bf16 tensors, CSR masks); no attention arithmetic.
  build      -- in-tree build of the HIP library and the host-side generator library.
"""
