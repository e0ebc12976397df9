"""CPU oracle of the quantized Adam step (test infrastructure only).

Nothing in the product imports this package.  See stq_oracle.c for the passages
of the paper each function follows.
"""
