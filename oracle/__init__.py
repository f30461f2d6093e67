"""TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.

Plain CPU oracle of the hybrid-cache decode step (see hybridkv_oracle.c).
"""
