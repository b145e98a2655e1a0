"""CPU oracle for the HALO group-sparse FFN path -- test infrastructure only.

Nothing in the product package may import this; see halo_ref.c for what it defines.
"""
