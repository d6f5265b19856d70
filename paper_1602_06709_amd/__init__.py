"""MI355X-native conv / FC / SGD training path (arxiv 1602.06709, Section 2).

`binding` is the thin ctypes layer over the C-ABI library `libcnn.so`;
`net` sequences its calls for the benchmark networks; `synth` holds the seeded
workload generators.  The GPU library is loaded on first use and its absence is
an error -- there is no CPU fallback.
"""
__all__ = ["binding", "net", "synth"]
