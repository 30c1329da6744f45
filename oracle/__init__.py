"""CPU oracle of the CQ hot path: TEST INFRASTRUCTURE (see cq_oracle.c's header).

Only tests, the smoke check and the bench's cpu_baseline leg may import this.
"""
