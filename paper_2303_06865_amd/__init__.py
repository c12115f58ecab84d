"""MI355X-native 4-bit group-wise OPT generation path (after FlexGen, arXiv 2303.06865).

The HIP library is loaded lazily by `paper_2303_06865_amd.binding`; importing this
package alone touches neither the GPU nor the shared library.
"""
__all__ = ["binding", "synth"]
