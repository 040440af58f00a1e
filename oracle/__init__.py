"""CPU oracle for the truncated quantizer (arXiv 2402.01798) -- TEST INFRASTRUCTURE.

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the GPU library.

``binding``  ctypes front end of ``tq_oracle.c`` (element-wise path, Sec. III-A, Alg. 1)
``params``   fp64 numpy statement of the parameter design (Sec. IV, Sec. V)
"""
