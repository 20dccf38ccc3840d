"""Segmented multi-adapter LoRA forward/backward for MI355X (gfx950): thin Python binding over the
C-ABI library in csrc/ plus the seeded synthetic workloads.  The binding is loaded lazily so that
`synth` can be used on machines without the built library; every compute entry point raises if
the HIP library is missing (there is no CPU fallback)."""

__all__ = ["synth", "binding"]
