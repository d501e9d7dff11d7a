"""CPU oracle of staleness-aware n-softsync ASGD -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It shares no code with the HIP path and never calls it.

  oracle.cnn       calcGradient of one learner (double precision, plain C loops)
  oracle.protocol  the parameter-server iteration (Sections 2.1, 2.2, 2.4, 3)
"""
from . import cnn, protocol  # noqa: F401
