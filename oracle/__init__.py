"""CPU oracle of the DMMV single-move descent.  TEST INFRASTRUCTURE ONLY.

Nothing in the GPU library or its Python binding imports this package.
"""
