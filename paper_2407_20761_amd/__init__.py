"""MI355X-native hot path of OmniBal-style balanced VLM training: packed variable-length
transformer-block forward/backward (hand-written gfx950 kernels behind a C ABI) and the host-side
balanced mini-batch packer.  This package only marshals arguments; all arithmetic runs in
libomnibal.so.  There is no CPU fallback: touching any entry point without the built library
raises ImportError.

The binding is loaded on first attribute access so that `paper_2407_20761_amd.build` can be
imported (to build the library) before the library exists."""
import importlib


def __getattr__(name):
    if name.startswith("__"):
        raise AttributeError(name)
    binding = importlib.import_module(".binding", __name__)
    return getattr(binding, name)
