"""Per-example gradient norms, clip factors and clipped gradient sums on MI355X.

`workloads` draws the seeded synthetic inputs; `dpclip` is the thin binding
over the C-ABI library built from `csrc/` (it raises if the library has not
been built).  Nothing here falls back to a CPU implementation.
"""
