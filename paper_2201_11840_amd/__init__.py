"""MI355X-native runtime for GC3-IR collective programs (interpreter, Section 6 of the paper)."""
