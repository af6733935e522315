"""Clustered vocabulary projection for MI355X (gfx950): package root."""
