"""MI355X-native AdamS / N:M hot path of CAST (arXiv 2509.25996).

``binding`` wraps the C-ABI library (``libcast.so``, hand-written HIP for gfx950) one to one;
``synth`` makes seeded synthetic inputs.  Importing the package loads nothing; the library
is loaded on first use and its absence is an error, never a fallback.
"""
