"""MI355X-native hot path of SketchedAMSGrad (gradient averaging, Alg. 2 of arXiv 2210.07454).

``paper_2210_07454_amd.sams`` is the thin binding over the C-ABI HIP library (loaded lazily);
``paper_2210_07454_amd.inputs`` holds the seeded synthetic input generators.
"""
__all__ = ["inputs", "sams"]
