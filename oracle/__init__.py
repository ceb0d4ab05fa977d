"""CPU oracle of the hybrid-cache decode attention step.  TEST INFRASTRUCTURE ONLY.

`apt_oracle.c` (built to `libapt_oracle.so` by `oracle/build.py`) evaluates the
paper's definitions in double precision; `oracle.py` is its ctypes loader;
`plan_oracle.py` is the plain statement of the work-partition rule.  Nothing here
imports or is imported by the GPU library.
"""
