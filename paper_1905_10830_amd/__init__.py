"""Feature-map transform coding (arXiv 1905.10830) on MI355X: thin Python
binding over the C-ABI library libfmtc.so (hand-written HIP for gfx950).

`paper_1905_10830_amd.binding` holds the calls (same names as the C entry
points, without the prefix); `paper_1905_10830_amd.synth` the seeded input
generators.  The library is loaded on first use; a missing library is an
error, there is no CPU fallback.
"""


def __getattr__(name):
    # binding is imported lazily so that the input generators can be used without torch
    if name == "binding":
        import importlib

        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
