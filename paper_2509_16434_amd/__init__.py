"""MI355X-native PPO learner hot path (experience buffer, GAE, clipped-PPO and
distillation minibatch updates of a depth-CNN + MLP actor-critic) behind a
C-ABI HIP library.  `learner` is the thin ctypes binding; `configs` and `synth`
hold the workload registry and the seeded input generators."""
from . import configs, synth  # noqa: F401

__all__ = ["configs", "synth", "learner"]


def __getattr__(name):
    if name == "learner":
        import importlib
        return importlib.import_module(".learner", __name__)
    raise AttributeError(name)
