"""MI355X-native hot path of Online Model Compression (OMC).

`paper_2205_03494_amd.omc` is the thin binding over the C-ABI library libomc (HIP kernels for
gfx950); `paper_2205_03494_amd.synth` generates the seeded synthetic inputs.  Importing the
package itself loads nothing native.
"""
__all__ = ["omc", "synth"]
