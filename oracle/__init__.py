"""CPU oracle for the extend / verify path.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's CPU-baseline leg may import this package; the
product path (the HIP library and its binding) never does, and shares no code with it.
"""
