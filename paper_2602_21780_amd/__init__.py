"""MI355X-native per-frame streaming step of XStreamVGGT (attend over a budgeted, quantized KV
cache → score → top-k prune → re-quantize), behind the C-ABI library libxsv.so.

`paper_2602_21780_amd.xsv` is the thin binding (argument marshalling only);
`paper_2602_21780_amd.inputs` generates the seeded synthetic streams.
"""
