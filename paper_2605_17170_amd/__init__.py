"""TriAxialKV decode / append hot path for AMD MI355X (gfx950)."""
