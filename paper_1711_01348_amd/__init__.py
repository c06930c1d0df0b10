"""MI355X-native evaluation of element-wise defined tensors and their gather-form gradients.

``workloads`` describes expressions and draws synthetic inputs (no arithmetic of the method);
``binding`` is the ctypes layer over libtad.so and is imported lazily so that the workload
descriptions can be used without the compiled library.
"""
_LAZY = ("binding", "Plan", "plan_derive", "eval_forward", "eval_backward", "TadError")


def __getattr__(name):
    if name in _LAZY:
        import importlib
        b = importlib.import_module(__name__ + ".binding")
        return b if name == "binding" else getattr(b, name)
    raise AttributeError(name)
