"""MI355X-native batch evaluator for reduction programs (the hot path of the P^2 synthesizer).

`workloads` describes the synthetic inputs; `binding` marshals arguments into the C-ABI
library built from csrc/ (imported on first use, fails loudly if the library is missing).
"""
from . import workloads  # noqa: F401


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
