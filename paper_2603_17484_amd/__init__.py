"""L2A token-wise conditional attention for MI355X (gfx950): hand-written HIP kernels behind a
C-ABI library (l2a_route_compact, l2a_attn_fwd, l2a_attn_bwd) and a thin ctypes binding."""
