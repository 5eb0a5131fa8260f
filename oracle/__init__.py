"""CPU oracle for the lookahead-step attention and greedy verification.

Test infrastructure only: nothing on the product path may import this package.
"""
