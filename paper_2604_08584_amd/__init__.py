"""CSAttention online-decode step for MI355X (gfx950): hand-written HIP kernels behind a C-ABI
library, with a thin ctypes binding (`binding`) and the seeded workload generator (`workload`)."""
