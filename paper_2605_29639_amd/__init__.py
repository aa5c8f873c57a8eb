"""Quantized KV-cache write and quantized paged decode attention for MI355X (gfx950).

`paper_2605_29639_amd.kvq` is the Python binding over the C-ABI library built from
`csrc/`; `paper_2605_29639_amd.workloads` draws the synthetic benchmark inputs.
"""
