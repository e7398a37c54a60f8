"""MI355X-native training-step library with performance-model-guided feature-map swapping.

`paper_1901_06773_amd.binding` is the ctypes binding of libaccudnn.so (built by
`paper_1901_06773_amd.build`).  The binding is imported on first use so that the
build step itself can import this package before the library exists.
"""


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
