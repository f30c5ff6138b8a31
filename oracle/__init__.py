"""CPU oracle of the DSFQ W4A4 linear layer (test infrastructure, not product code).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
See dsfq_oracle.c for the definitions and citations; this module only marshals
numpy arrays to that C code and strings its steps together in the paper's order.
"""
from .dsfq import *  # noqa: F401,F403
from . import nfds  # noqa: F401,E402  (calibration-set arithmetic of Sec. 3.3)
from . import calib  # noqa: F401,E402  (learnable smoothing factor and steps: the layer-wise reconstruction loss and its derivatives)
