"""MI355X-native local computation of one TED Mixture-of-Experts layer (HIP, gfx950).

The GPU library is loaded lazily by :mod:`paper_2303_06318_amd.moe`; importing the package
(or :mod:`paper_2303_06318_amd.synth`) does not need a GPU.
"""
