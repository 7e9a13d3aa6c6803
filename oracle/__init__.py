"""CPU oracle for ADSA decode -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It never imports the HIP package and the HIP package never imports it.
"""
from .adsa_oracle import (  # noqa: F401
    OracleCfg, build, classify, vcos, rank_keep, budget, select, attend,
    accumulate, compact, step, CacheState, make_cfg, PREFIX, LOCAL, CANDIDATE,
)
