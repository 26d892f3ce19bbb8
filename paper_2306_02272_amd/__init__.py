"""OWQ mixed-precision linear layer on MI355X: thin Python binding over libowq.so.

Importing the package loads nothing; `paper_2306_02272_amd.binding` opens the
shared library on first use and raises if it has not been built.
"""
__all__ = ["binding", "build"]
