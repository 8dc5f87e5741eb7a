"""dcpq: two-pass product-quantization search with derived codebooks, native on MI355X (gfx950).

The product is the C-ABI library built from ``csrc/`` (declared in ``include/dcpq.h``); the
Python side is argument marshalling only (``binding``) plus seeded input generators (``synth``).
"""
