"""MI355X-native fp32 operator kernels for the workloads of arXiv 2006.06762.

``paper_2006_06762_amd.inputs`` (seeded synthetic tensors) imports without the
HIP library; everything else is the ctypes binding of ``libanr.so`` and is
loaded on first use.  If the library has not been built, that first use raises.
"""
import importlib

from . import inputs  # noqa: F401


def __getattr__(name):
    # Lazy: keep `import paper_2006_06762_amd.inputs` free of the HIP library.
    if name.startswith("__"):
        raise AttributeError(name)
    if name == "build":
        # the build script must import in a tree that has no built library yet
        return importlib.import_module(__name__ + ".build")
    binding = importlib.import_module(__name__ + ".binding")
    if name == "binding":
        return binding
    if hasattr(binding, name):
        return getattr(binding, name)
    raise AttributeError("module %r has no attribute %r" % (__name__, name))
