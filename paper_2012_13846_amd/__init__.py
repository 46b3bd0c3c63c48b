"""MI355X-native generalized sparse convolution (coordinate hashing, kernel maps, conv fwd/dgrad/wgrad).

`spgen` (synthetic inputs) is importable anywhere.  The HIP path is reached through
`paper_2012_13846_amd.binding`, which loads the in-tree C-ABI library and raises if it
is missing: there is no CPU fallback.
"""
__all__ = ["spgen", "binding"]
