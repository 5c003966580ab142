"""Measurement aids of ``bench.py``: timing loops on the C side of the library's
boundary and a comparison program for the runtime's own batched copy call.
Not part of the library: nothing under ``paper_2511_06605_amd`` uses this."""
