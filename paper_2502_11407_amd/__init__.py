"""MI355X-native scheduled dense operators (GEMM, batched matmul, conv2d) and the
graph-walk schedule constructor.  The compute path lives in csrc/ behind a C ABI
(include/gensor.h); `binding` marshals arguments to it.  Importing the package does
not load the library; the first use of a binding name does, and fails loudly if it
has not been built."""

_BINDING_NAMES = None


def __getattr__(name):
    if name in ("inputs", "binding"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    from . import binding
    if hasattr(binding, name):
        return getattr(binding, name)
    raise AttributeError(name)
