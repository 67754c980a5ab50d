"""Runs the CPU boundary tests against a given build of the library's host side (the sanitizer
build): every load of libuniprefill.so in this process is redirected to that file.  Test
infrastructure only -- the package itself knows no such switch."""
import ctypes
import os
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
sanitized = os.path.abspath(sys.argv[1])
_real = ctypes.CDLL


class _Redirect(_real):
    def __init__(self, name, *args, **kwargs):
        if name is not None and os.path.basename(str(name)) == "libuniprefill.so":
            name = sanitized
        super().__init__(name, *args, **kwargs)


ctypes.CDLL = _Redirect
sys.exit(pytest.main([os.path.join(os.path.dirname(HERE), "test_host_boundary.py"), "-q", "-x", "-p", "no:cacheprovider"]))
