"""The GPU parity tests' view of the package's emulated-rank plumbing (device buffers, streams,
calls through the binding).  Nothing is defined here."""
from paper_2604_24013_amd.emulated_rank import *  # noqa: F401,F403
