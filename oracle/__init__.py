"""fp64 CPU oracle of the QuickPrefill path. Test infrastructure only; see qp_oracle.py."""
from .qp_oracle import *  # noqa: F401,F403
