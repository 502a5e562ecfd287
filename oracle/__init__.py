"""CPU oracle for the Slide Attention operator -- test infrastructure only.

Nothing in the product package imports this.  See slide_oracle.c for what it
computes and which passages of the paper it follows.
"""
