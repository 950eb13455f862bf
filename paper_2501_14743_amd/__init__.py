"""MI355X-native paged KV-cache pull (the KV transfer data path of KVDirect, arXiv 2501.14743).

``paper_2501_14743_amd.kvd`` is the thin binding over the C ABI declared in ``include/kvd.h``;
``paper_2501_14743_amd.workloads`` generates the seeded synthetic inputs.  Nothing is loaded
at import time; the first call into ``kvd`` loads ``libkvd.so`` and fails loudly if it is
missing.
"""
