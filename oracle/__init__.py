"""fp64 CPU oracle for the DBSA attention path -- test infrastructure only.

Nothing under the product package imports this; it shares no code with the
HIP library.  See dbsa_oracle.py (attention) and layout_oracle.py (tile lists).
"""
