"""MI355X-native SlimFit hot path (freeze score, activation codec, score pruning, ILS).

``paper_2305_18513_amd.binding`` wraps the C-ABI library built from ``csrc/``;
``paper_2305_18513_amd.synth`` draws the seeded synthetic workloads.  Importing
the package loads nothing native; the binding loads the library on first use
and raises if it has not been built.
"""
