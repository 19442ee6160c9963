"""CPU oracle for the ASER calibration path.  Test infrastructure only: nothing on the
product path may import this package (see aser_oracle.py's header)."""
