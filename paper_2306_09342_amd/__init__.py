"""MI355X-native reversible-stack backward (Reprop / PaReprop schedules).

The compute lives in the C-ABI library built from ``csrc/``; ``binding`` only
marshals arguments.  ``synth`` draws the seeded synthetic workloads.
"""
