"""MI355X-native CodedReduce hot path: thin ctypes binding over libcodedreduce.so (argument marshalling only)."""
from .api import *  # noqa: F401,F403
