"""CPU oracle for the capsule-convolution forward pass.  Test infrastructure only.

Nothing in the product package imports this; only the tests, the smoke check and the
CPU-baseline leg of the bench do.
"""
