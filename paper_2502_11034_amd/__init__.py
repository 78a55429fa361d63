"""MI355X-native fused AdaGC + AdamW/Lion optimizer step (arxiv 2502.11034).

`binding` loads the HIP library and mirrors its C entry points; `workloads`
produces seeded synthetic inputs and contains none of the method's arithmetic.
Importing the package loads nothing; the library is opened on first use.
"""
