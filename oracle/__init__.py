"""CPU oracle of the DSV sparse-attention path.  Test infrastructure only.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package; the product package never does.
"""
from .dsv_oracle import *  # noqa: F401,F403
