"""Predictive delta coding of transformer KV caches on MI355X (gfx950).

`plc` holds the thin binding over the C-ABI device library (libplc.so);
`workloads` draws the seeded synthetic inputs.  The device library is the only
implementation: there is no CPU fallback, and calls fail loudly when it is
missing.
"""
