"""CPU oracle and reference models -- test infrastructure only.

Nothing under this package is part of the product path: the HIP library and its
Python binding never import it, and it never imports them.
"""
