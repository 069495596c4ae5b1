"""MI355X-native H2O (Heavy-Hitter Oracle) attention hot path.

`binding` exposes the C-ABI library (libh2o_hip.so); `synth` holds the seeded
synthetic input generators shared by tests and benchmark.  The library must be
built first (`python -m paper_2306_14048_amd.build`); there is no fallback.
"""
