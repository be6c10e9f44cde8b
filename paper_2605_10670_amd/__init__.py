"""Membership-elastic MoE dispatch/combine for AMD MI355X (gfx950).

`binding` wraps the C-ABI library (include/eep.h); `synth` makes seeded inputs.
"""
