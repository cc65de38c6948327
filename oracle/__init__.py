"""CPU oracle for Double Sparsity decode attention -- test infrastructure only.

Nothing under this folder is part of the product path; the product package never
imports it.  See ds_oracle.c for the statement of what is computed.
"""
