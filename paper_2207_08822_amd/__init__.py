"""Integer (dynamic fixed-point) linear-layer step on MI355X: see fxp.py."""
