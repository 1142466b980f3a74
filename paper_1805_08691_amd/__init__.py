"""MI355X-native int8 quantised convolution (the hot path of arxiv 1805.08691).

``paper_1805_08691_amd.binding`` is a thin ctypes layer over ``libq8conv.so`` (C ABI in
``include/q8conv.h``); ``workloads`` holds seeded synthetic inputs and layer lists.
Nothing is imported eagerly so that the input generators can be used without the library.
"""
__all__ = ["binding", "workloads", "build"]
