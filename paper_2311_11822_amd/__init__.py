"""MI355X-native Book-Keeping clipped-gradient path: thin Python binding over libdp_bk.so.

Every step of the path runs in the library's HIP kernels; this package only marshals
arguments.  Importing `paper_2311_11822_amd.binding` raises if the library has not been
built (python -m paper_2311_11822_amd.build): there is no fallback path.
"""
