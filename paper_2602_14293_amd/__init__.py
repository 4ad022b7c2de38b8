"""MI355X-native knowledge-base retrieval (cosine scoring, tag filter, top-k) behind a C ABI.

Importing the package loads nothing native; ``paper_2602_14293_amd.kb`` loads ``libkb.so`` on
first use and raises if it has not been built.
"""
