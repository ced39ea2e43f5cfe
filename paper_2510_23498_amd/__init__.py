"""MI355X-native mixed-precision neural-ODE time stepping (forward + discrete adjoint).

The compute path lives in the HIP library under ``csrc/`` behind a C ABI
(see ``include/rampde.h``); ``binding`` marshals arguments to it.  Importing this
package does not load the library: the first call does, and fails loudly if it
has not been built.
"""
from . import workloads  # noqa: F401
