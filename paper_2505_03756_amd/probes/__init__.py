"""Hardware probes behind the design notes of the attention kernel (not part of the product path).

`python -m paper_2505_03756_amd.probes` builds and runs issue_power_probe.hip (needs hipcc and a
gfx950 GPU); `python -m paper_2505_03756_amd.probes --per-tile` times the library's own attention
kernel per 64-key tile step on a few and on all CUs.
"""
