"""libgaf: Gradient Agreement Filtering aggregation on MI355X (gfx950)."""
