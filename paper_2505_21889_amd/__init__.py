"""EFIM cache-hit extend attention for AMD MI355X (gfx950)."""
