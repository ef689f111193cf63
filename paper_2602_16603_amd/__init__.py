"""MI355X-native op-preemptible prefill (FlowPrefill hot path).

`binding` wraps the C-ABI library `libflowprefill.so` (hand-written HIP kernels for gfx950);
`inputs` draws the seeded synthetic workloads; `eventloop` is the minimal arrival/completion
driver.  Nothing is imported eagerly so that the input generators can be used without the
compiled library; using `binding` without the library raises.
"""
__all__ = ["binding", "inputs", "eventloop"]
