"""MI355X-native mixed-batch paged attention + KV block swap (ProServe engine step).

Importing the package loads nothing native; ``paper_2512_12928_amd.binding`` loads the
C-ABI shared library and raises if it has not been built.
"""
__all__ = ["workloads", "binding"]
