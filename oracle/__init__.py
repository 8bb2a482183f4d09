"""CPU oracle for the deduplicated expert-parallel MoE layer.

TEST INFRASTRUCTURE ONLY: a plain, slow, independent restatement of what the layer computes,
written from the paper.  Only tests/, the smoke check and the benchmark's cpu_baseline leg may
import it; the product package never does, and the two share no code.
"""
