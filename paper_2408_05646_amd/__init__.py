"""Eigen Attention low-rank inference path for MI355X (gfx950)."""
