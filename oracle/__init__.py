"""Test infrastructure only: the plain fp64 CPU oracle of the draft / verify / accept path.

Nothing in the product package imports this directory.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may call it.
"""
