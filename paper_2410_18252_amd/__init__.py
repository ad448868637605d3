"""MI355X-native generation hot path of asynchronous online-DPO RLHF (librlgen.so + ctypes binding).

Importing the package does not load the library; `paper_2410_18252_amd.rlgen` does, and fails
loudly if it has not been built (python -m paper_2410_18252_amd.build).
"""
