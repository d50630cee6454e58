"""CPU oracle for the GALA linear layers -- test infrastructure only.

Nothing in the product package imports this.  See ``gala_oracle.c`` for the
arithmetic; ``oracle.py`` is a ctypes wrapper that only marshals numpy arrays.
"""
