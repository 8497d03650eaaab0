"""MI355X-native NAV (non-autoregressive verification) pass of PipeSD's cloud side.

`inputs` draws seeded synthetic workloads; `nav` is the thin binding over the C-ABI HIP
library (importing it fails loudly when the library has not been built)."""
