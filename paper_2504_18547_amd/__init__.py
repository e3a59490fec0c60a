"""Integerized ViT block matmuls (operand reordering) for MI355X: Python binding of libvitq."""
