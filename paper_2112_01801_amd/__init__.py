"""SH continuous-filter mesh convolutions (facet2vertex, vertex2facet, facet2facet) for MI355X.

`meshgen` (pure numpy input generators) imports without a GPU; the HIP library is loaded on
first use of `binding`.
"""
__all__ = ["meshgen", "binding"]
