"""Gram-threshold representative-token selection and the cascade step for MI355X (gfx950)."""
