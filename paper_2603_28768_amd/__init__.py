"""MI355X-native MoE rank-forward path under a CRAFT replication plan.

`binding` wraps the C-ABI library (`libcraft.so`, built from `csrc/`); `synth`
draws the seeded synthetic inputs.  Importing the package loads nothing native.
"""
