"""MI355X-native forward pass of one EdgeShard shard (a contiguous range of Llama2 decoder
layers).  `binding` wraps the C-ABI of libshard.so; `synth` draws seeded synthetic inputs."""
from . import synth  # noqa: F401


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
