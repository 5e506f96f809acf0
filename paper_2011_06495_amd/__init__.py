"""Majority-voting sparse-SGD vote step on MI355X (gfx950).

`paper_2011_06495_amd.binding` is the thin ctypes layer over the C-ABI
library (mv_begin / mv_vote_step / mv_end); `paper_2011_06495_amd.workloads`
draws the seeded synthetic inputs.  Nothing is loaded at import time.
"""
