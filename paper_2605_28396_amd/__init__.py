"""libadwin_opd: MI355X-native teacher-anchored per-token supervision for on-policy
distillation over ragged student rollouts (thin Python binding over a C-ABI library)."""

__all__ = ["synth"]
