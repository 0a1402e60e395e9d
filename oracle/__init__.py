"""CPU oracle for the co-serving attention / KV-cache hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import, call, link or
execute anything in this directory; only the tests, the smoke check and the benchmark's
CPU-baseline leg do.  The oracle shares no code, header, table or helper with the HIP
library and never imports it.

* ``attention``  -- fp64 softmax attention over the logical (unpaged) sequence
                    (C, ``cs_oracle.c``, called through ctypes).
* ``kv_layout``  -- the KV-pool format written out as index arithmetic, and the reference
                    append / checkpoint-gather / restore copies over it (numpy).
"""
