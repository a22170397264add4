"""MI355X-native transformer-layer training step (the layer a Slapo schedule produces).

The arithmetic lives entirely in the HIP library ``libslapo_mi355x.so``; this package is a thin
ctypes binding (argument marshalling only). Import :mod:`paper_2302_08005_amd.binding` to use it.
"""
