"""Plain CPU reference for the streaming-rollout frame update.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product path never imports it and shares no
code with it.
"""
