"""MI355X-native hot path of the Dolphin neurosymbolic framework (arXiv 2410.03348).

``paper_2410_03348_amd.binding`` is the ctypes front of ``libdolphin_hip.so``
(hand-written HIP kernels for gfx950 behind the C ABI of ``include/dolphin_hip.h``);
``paper_2410_03348_amd.programs`` composes its calls into the benchmark programs;
``paper_2410_03348_amd.build`` compiles the library in-tree.  Importing the binding
without a built library raises ImportError: there is no CPU fallback.
"""
__version__ = "0.1.0"
