"""MI355X-native 4-bit quantized GEMM / im2col convolution (libq4).

``paper_2009_06488_amd.q4`` is the thin binding over the C-ABI library;
``paper_2009_06488_amd.workloads`` draws the seeded synthetic inputs.
The binding is imported lazily so that the input generators can be used
without the GPU library.
"""


def __getattr__(name):
    if name == "q4":
        import importlib
        return importlib.import_module(".q4", __name__)
    raise AttributeError(name)
